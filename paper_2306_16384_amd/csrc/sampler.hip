// GPU neighbourhood sampler over a CSR graph (GIDS paper, Section 2.2.2:
// GraphSAGE-style sampling of up to `fanout` neighbours per node per layer,
// uniformly at random; Section 3.5: the structure data is small next to the
// features and is sampled by GPU threads directly, from GPU memory or zero-copy
// from pinned CPU memory).  It produces the raw node-ID list that the window
// push and the gather take, without a trip to the host.
//
// Sampling law (the same counter-based hashing the synthetic workloads use, so
// that a CPU implementation reproduces every list bit for bit):
//   mix64(z): z ^= z >> 30; z *= 0xBF58476D1CE4E5B9; z ^= z >> 27; z *= 0x94D049BB133111EB; z ^= z >> 31
//   H(seed, tag, x1..xk): k = mix64(seed + tag * 0x9E3779B97F4A7C15); k = mix64(k ^ xi) for each xi
//   seed node i of minibatch b:  H(seed, 4, b, i) mod n_nodes      (or Zipf-ranked, see seeds_kernel)
//   hop l expands the distinct nodes hop l-1 produced (hop 0: the distinct seeds), ascending;
//   node v of degree d with fanout f: d <= f -> all d neighbours in slot order; else f distinct
//   slots by Floyd's subset sampling: for j = d-f .. d-1: t = H(seed, 5, b, l, v, j) mod (j+1),
//   take t unless already taken, else j; neighbours are emitted in draw order.
// Output = seeds, then each hop's neighbours in (node ascending, draw) order, duplicates kept.
//
// Per hop: `take` counts min(d, f) per frontier node and the last workgroup
// turns workgroup sums into offsets (so every node knows where its neighbours
// go), `sample` draws and writes, then the hop's output is deduplicated into
// the next frontier with the bitmap kernels of dedup.hip.
#include <algorithm>

#include "gids_dev.h"
#include "scan.h"

namespace gids {

namespace {

constexpr int SM_THREADS = SCAN_THREADS;
constexpr uint64_t GOLDEN = 0x9E3779B97F4A7C15ull;

__host__ __device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

template <typename IdT>
__global__ void seeds_kernel(uint64_t ks, uint64_t n_seeds, uint64_t n_nodes, const uint64_t* __restrict__ rank_table,
                             uint64_t perm_mult, uint64_t perm_add, IdT* __restrict__ raw, SamplerState* st) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) {
        st->n_raw = (uint32_t)n_seeds;
        st->layer_count = (uint32_t)n_seeds;
    }
    if (i >= n_seeds) return;
    const uint64_t h = mix64(ks ^ i);
    if (!rank_table) {
        raw[i] = (IdT)(h % n_nodes);
        return;
    }
    // Zipf-ranked seeds: rank = number of cumulative thresholds <= (h >> 1); node = (rank * mult + add) mod n
    const uint64_t u = h >> 1;
    uint64_t lo = 0, hi = n_nodes;
    while (lo < hi) {
        const uint64_t mid = lo + (hi - lo) / 2;
        if (rank_table[mid] <= u) lo = mid + 1; else hi = mid;
    }
    const uint64_t r = lo < n_nodes - 1 ? lo : n_nodes - 1;
    raw[i] = (IdT)((r * perm_mult + perm_add) % n_nodes);      // n_nodes < 2^31 is checked by the host: no overflow
}

template <typename IdT>
__global__ __launch_bounds__(SM_THREADS) void take_kernel(const IdT* __restrict__ frontier,
                                                          const uint32_t* __restrict__ n_front_ptr,
                                                          const int64_t* __restrict__ indptr, uint32_t fanout,
                                                          uint32_t* blocksum, uint32_t* blockoff, SamplerState* st) {
    __shared__ uint32_t smem[8];
    __shared__ uint32_t is_last;
    __shared__ uint32_t running;
    const uint32_t n_front = *n_front_ptr;
    const uint64_t i = (uint64_t)blockIdx.x * SM_THREADS + threadIdx.x;
    uint32_t take = 0;
    if (i < n_front) {
        const uint64_t v = (uint64_t)frontier[i];
        const int64_t deg = indptr[v + 1] - indptr[v];
        take = deg < (int64_t)fanout ? (uint32_t)deg : fanout;
    }
    uint32_t total;
    block_exclusive_scan(take, &total, smem);
    if (threadIdx.x == 0) {
        __hip_atomic_store(&blocksum[blockIdx.x], total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __threadfence();
        const uint32_t tk = atomicAdd(&st->ticket, 1u);
        is_last = (tk == gridDim.x - 1);
        running = 0;
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();
    const uint32_t nb = gridDim.x;
    for (uint32_t base = 0; base < nb; base += SM_THREADS) {
        const uint32_t b = base + threadIdx.x;
        const uint32_t x = b < nb ? __hip_atomic_load(&blocksum[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
        uint32_t chunk;
        const uint32_t excl = block_exclusive_scan(x, &chunk, smem);
        if (b < nb) blockoff[b] = running + excl;
        __syncthreads();
        if (threadIdx.x == 0) running += chunk;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        st->layer_base = st->n_raw;        // this hop's neighbours go behind everything sampled so far
        st->layer_count = running;
        st->n_raw += running;
        st->ticket = 0;
    }
}

template <typename IdT>
__global__ __launch_bounds__(SM_THREADS) void sample_kernel(const IdT* __restrict__ frontier,
                                                            const uint32_t* __restrict__ n_front_ptr,
                                                            const int64_t* __restrict__ indptr,
                                                            const IdT* __restrict__ indices, uint32_t fanout, uint64_t kl,
                                                            const uint32_t* __restrict__ blockoff,
                                                            IdT* __restrict__ raw, IdT* __restrict__ hop_out,
                                                            const SamplerState* st) {
    __shared__ uint32_t smem[8];
    const uint32_t n_front = *n_front_ptr;
    const uint64_t i = (uint64_t)blockIdx.x * SM_THREADS + threadIdx.x;
    uint64_t v = 0;
    int64_t start = 0, deg = 0;
    uint32_t take = 0;
    if (i < n_front) {
        v = (uint64_t)frontier[i];
        start = indptr[v];
        deg = indptr[v + 1] - start;
        take = deg < (int64_t)fanout ? (uint32_t)deg : fanout;
    }
    uint32_t total;
    const uint32_t pos = blockoff[blockIdx.x] + block_exclusive_scan(take, &total, smem);
    if (take == 0) return;
    IdT* dst_raw = raw + st->layer_base + pos;
    IdT* dst_hop = hop_out + pos;
    if (deg <= (int64_t)fanout) {
        for (uint32_t s = 0; s < take; s++) {
            const IdT nb = indices[start + s];
            dst_raw[s] = nb;
            dst_hop[s] = nb;
        }
        return;
    }
    const uint64_t kv = mix64(kl ^ v);
    uint32_t chosen[64];                   // fanout <= 64 (checked by the host); slots of one node fit 32 bits
    uint32_t m = 0;
    for (int64_t j = deg - fanout; j < deg; j++) {
        uint32_t t = (uint32_t)(mix64(kv ^ (uint64_t)j) % (uint64_t)(j + 1));
        bool seen = false;
        for (uint32_t c = 0; c < m; c++) seen |= (chosen[c] == t);
        if (seen) t = (uint32_t)j;
        chosen[m] = t;
        const IdT nb = indices[start + t];
        dst_raw[m] = nb;
        dst_hop[m] = nb;
        m++;
    }
}

// ---- expected visits per node (hot-node ranking) ---------------------------
// lam_0 = n_seeds / n for every node; a node expected c = min(1, lam_l) times in hop l's frontier sends
// w = c * min(deg, f_l) / deg along each adjacency slot; score = sum of lam over the hops.  32.32 fixed
// point, floor divisions, 64-bit integer atomics: the sums do not depend on the order of the additions.

__global__ void visits_init_kernel(uint64_t* __restrict__ cur, uint64_t* __restrict__ score, uint64_t n, uint64_t lam0) {
    for (uint64_t v = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += (uint64_t)gridDim.x * blockDim.x) {
        cur[v] = lam0;
        score[v] = lam0;
    }
}

// one wavefront per node: lanes stride over the node's adjacency slots
template <typename IdT>
__global__ __launch_bounds__(SM_THREADS) void visits_hop_kernel(const int64_t* __restrict__ indptr,
                                                                const IdT* __restrict__ indices, uint64_t n,
                                                                uint64_t fanout, const uint64_t* __restrict__ cur,
                                                                unsigned long long* __restrict__ nxt) {
    const uint64_t ONE = 1ull << 32;
    const uint64_t wave0 = ((uint64_t)blockIdx.x * SM_THREADS + threadIdx.x) >> 6;
    const uint64_t n_waves = ((uint64_t)gridDim.x * SM_THREADS) >> 6;
    for (uint64_t v = wave0; v < n; v += n_waves) {
        const uint64_t lam = cur[v];
        const int64_t start = indptr[v];
        const uint64_t deg = (uint64_t)(indptr[v + 1] - start);
        if (!lam || !deg) continue;
        const uint64_t c = lam < ONE ? lam : ONE;
        const uint64_t take = deg < fanout ? deg : fanout;
        const uint64_t w = c * take / deg;
        if (!w) continue;
        for (uint64_t s = lane_id(); s < deg; s += 64) atomicAdd(&nxt[(uint64_t)indices[start + s]], (unsigned long long)w);
    }
}

__global__ void visits_add_kernel(uint64_t* __restrict__ score, const uint64_t* __restrict__ nxt, uint64_t n) {
    for (uint64_t v = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += (uint64_t)gridDim.x * blockDim.x)
        score[v] += nxt[v];
}

__global__ void visits_zero_kernel(uint64_t* __restrict__ p, uint64_t n) {
    for (uint64_t v = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += (uint64_t)gridDim.x * blockDim.x)
        p[v] = 0;
}

// ---- weighted reverse PageRank (hot-node ranking, Section 3.3) ---------------
// r_(k+1)(u) = teleport + sum over adjacency slots v -> u of floor(floor(r_k(v) * damping / 65536) / deg v),
// total mass 2^44, integer atomics.

__global__ void rank_fill_kernel(uint64_t* __restrict__ p, uint64_t n, uint64_t value) {
    for (uint64_t v = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += (uint64_t)gridDim.x * blockDim.x)
        p[v] = value;
}

template <typename IdT>
__global__ __launch_bounds__(SM_THREADS) void rank_step_kernel(const int64_t* __restrict__ indptr,
                                                               const IdT* __restrict__ indices, uint64_t n,
                                                               uint64_t damping_q16, const uint64_t* __restrict__ cur,
                                                               unsigned long long* __restrict__ nxt) {
    const uint64_t wave0 = ((uint64_t)blockIdx.x * SM_THREADS + threadIdx.x) >> 6;
    const uint64_t n_waves = ((uint64_t)gridDim.x * SM_THREADS) >> 6;
    for (uint64_t v = wave0; v < n; v += n_waves) {
        const int64_t start = indptr[v];
        const uint64_t deg = (uint64_t)(indptr[v + 1] - start);
        if (!deg) continue;
        const uint64_t w = (cur[v] * damping_q16 >> 16) / deg;
        if (!w) continue;
        for (uint64_t s = lane_id(); s < deg; s += 64) atomicAdd(&nxt[(uint64_t)indices[start + s]], (unsigned long long)w);
    }
}

}  // namespace

template <typename IdT>
void launch_reverse_pagerank(const int64_t* indptr, const IdT* indices, uint64_t n, uint32_t damping_q16,
                             uint32_t n_iters, uint64_t* scratch, uint64_t* score, hipStream_t s) {
    const uint32_t flat = (uint32_t)std::min<uint64_t>((n + 255) / 256, 4096);
    const uint32_t per_node = (uint32_t)std::min<uint64_t>((n + 3) / 4, 1u << 16);
    const uint64_t base = (1ull << 44) / n;
    const uint64_t teleport = base * (65536u - damping_q16) >> 16;
    // ping-pong so that the last iteration lands in score[]
    uint64_t* cur = (n_iters & 1) ? scratch : score;
    uint64_t* nxt = (n_iters & 1) ? score : scratch;
    hipLaunchKernelGGL(rank_fill_kernel, dim3(flat), dim3(256), 0, s, cur, n, base);
    for (uint32_t k = 0; k < n_iters; k++) {
        hipLaunchKernelGGL(rank_fill_kernel, dim3(flat), dim3(256), 0, s, nxt, n, teleport);
        hipLaunchKernelGGL(rank_step_kernel<IdT>, dim3(per_node), dim3(SM_THREADS), 0, s, indptr, indices, n,
                           (uint64_t)damping_q16, cur, reinterpret_cast<unsigned long long*>(nxt));
        std::swap(cur, nxt);
    }
}

template <typename IdT>
void launch_visit_scores(const int64_t* indptr, const IdT* indices, uint64_t n, const uint32_t* fanouts,
                         uint32_t n_layers, uint64_t n_seeds, uint64_t* cur, uint64_t* nxt, uint64_t* score,
                         hipStream_t s) {
    const uint32_t flat = (uint32_t)std::min<uint64_t>((n + 255) / 256, 4096);
    const uint32_t per_node = (uint32_t)std::min<uint64_t>((n + 3) / 4, 1u << 16);
    hipLaunchKernelGGL(visits_init_kernel, dim3(flat), dim3(256), 0, s, cur, score, n, (n_seeds << 32) / n);
    for (uint32_t l = 0; l < n_layers; l++) {
        hipLaunchKernelGGL(visits_zero_kernel, dim3(flat), dim3(256), 0, s, nxt, n);
        hipLaunchKernelGGL(visits_hop_kernel<IdT>, dim3(per_node), dim3(SM_THREADS), 0, s, indptr, indices, n,
                           (uint64_t)fanouts[l], cur, reinterpret_cast<unsigned long long*>(nxt));
        hipLaunchKernelGGL(visits_add_kernel, dim3(flat), dim3(256), 0, s, score, nxt, n);
        std::swap(cur, nxt);
    }
}

uint64_t sampler_key(uint64_t seed, uint64_t tag) { return mix64(seed + tag * GOLDEN); }
uint64_t sampler_mix(uint64_t z) { return mix64(z); }

template <typename IdT>
void launch_seeds(uint64_t ks, uint64_t n_seeds, uint64_t n_nodes, const uint64_t* rank_table, uint64_t perm_mult,
                  uint64_t perm_add, IdT* raw, SamplerState* st, hipStream_t s) {
    const uint32_t grid = (uint32_t)((n_seeds + 255) / 256) + (n_seeds == 0);
    hipLaunchKernelGGL(seeds_kernel<IdT>, dim3(grid), dim3(256), 0, s, ks, n_seeds, n_nodes, rank_table, perm_mult,
                       perm_add, raw, st);
}

template <typename IdT>
void launch_hop(const IdT* frontier, const uint32_t* n_front, uint64_t front_upper, const int64_t* indptr,
                const IdT* indices, uint32_t fanout, uint64_t kl, uint32_t* blocksum, uint32_t* blockoff, IdT* raw,
                IdT* hop_out, SamplerState* st, hipStream_t s) {
    const uint32_t grid = (uint32_t)((front_upper + SM_THREADS - 1) / SM_THREADS) + (front_upper == 0);
    hipLaunchKernelGGL(take_kernel<IdT>, dim3(grid), dim3(SM_THREADS), 0, s, frontier, n_front, indptr, fanout,
                       blocksum, blockoff, st);
    hipLaunchKernelGGL(sample_kernel<IdT>, dim3(grid), dim3(SM_THREADS), 0, s, frontier, n_front, indptr, indices,
                       fanout, kl, blockoff, raw, hop_out, st);
}

#define GIDS_INSTANTIATE(IdT)                                                                                     \
    template void launch_seeds<IdT>(uint64_t, uint64_t, uint64_t, const uint64_t*, uint64_t, uint64_t, IdT*,      \
                                    SamplerState*, hipStream_t);                                                  \
    template void launch_visit_scores<IdT>(const int64_t*, const IdT*, uint64_t, const uint32_t*, uint32_t,      \
                                           uint64_t, uint64_t*, uint64_t*, uint64_t*, hipStream_t);              \
    template void launch_reverse_pagerank<IdT>(const int64_t*, const IdT*, uint64_t, uint32_t, uint32_t, uint64_t*, \
                                               uint64_t*, hipStream_t);                                          \
    template void launch_hop<IdT>(const IdT*, const uint32_t*, uint64_t, const int64_t*, const IdT*, uint32_t,    \
                                  uint64_t, uint32_t*, uint32_t*, IdT*, IdT*, SamplerState*, hipStream_t);
GIDS_INSTANTIATE(int32_t)
GIDS_INSTANTIATE(int64_t)

}  // namespace gids
