// ID dedup + sort for one minibatch (the node-ID list a neighbourhood sampler
// hands to feature aggregation, Sections 2.2.2-2.2.3 of the GIDS paper, holds
// every sampled neighbour, so hub nodes repeat thousands of times).
//
// The ID universe is the store's row count, so "sort + unique" is a bitmap:
//   mark   every workgroup filters its share of the raw list through an LDS
//          hash set (repeats of a hub collapse in LDS), survivors set one bit
//          each in a global bitmap of n_rows bits;
//   count  popcount per 1024-word block; the last block to arrive turns the
//          block sums into exclusive offsets and publishes the distinct count;
//   emit   every block rescans its words and writes the set bit positions at
//          its offset: the output is the ascending distinct ID list.
// No comparison sort, no global hash table, deterministic output.
#include "gids_dev.h"
#include "scan.h"

namespace gids {

namespace {

constexpr int DD_THREADS = SCAN_THREADS;
constexpr int MARK_ITEMS = 4;            // raw IDs per thread per tile
constexpr int TAB_LOG = 11;              // LDS hash set: 2048 slots x 8 B = 16 KiB
constexpr int TAB_SLOTS = 1 << TAB_LOG;
constexpr int TAB_PROBES = 4;
constexpr unsigned long long TAB_EMPTY = ~0ull;
constexpr int WORDS_PER_THREAD = 4;
constexpr int WORDS_PER_BLOCK = DD_THREADS * WORDS_PER_THREAD;

template <typename IdT>
__global__ __launch_bounds__(DD_THREADS) void mark_kernel(const IdT* __restrict__ ids, uint64_t n,
                                                          const uint32_t* __restrict__ n_dev, uint64_t n_rows,
                                                          uint64_t* __restrict__ bitmap, Ctl* ctl) {
    __shared__ unsigned long long tab[TAB_SLOTS];
    if (n_dev) n = *n_dev;                // the list's length is only known on the device (n was its bound)
    __shared__ uint32_t fresh_total;
    for (int i = threadIdx.x; i < TAB_SLOTS; i += DD_THREADS) tab[i] = TAB_EMPTY;
    if (threadIdx.x == 0) fresh_total = 0;
    __syncthreads();
    const uint64_t tile = (uint64_t)DD_THREADS * MARK_ITEMS;
    bool bad = false;
    for (uint64_t base = (uint64_t)blockIdx.x * tile; base < n; base += (uint64_t)gridDim.x * tile) {
        uint32_t fresh = 0;
#pragma unroll
        for (int k = 0; k < MARK_ITEMS; k++) {
            const uint64_t i = base + (uint64_t)k * DD_THREADS + threadIdx.x;
            if (i >= n) continue;
            const IdT raw = ids[i];
            if (raw < 0 || (uint64_t)raw >= n_rows) { bad = true; continue; }
            const unsigned long long v = (unsigned long long)raw;
            uint32_t h = (uint32_t)((v * 0x9E3779B97F4A7C15ull) >> (64 - TAB_LOG));
            bool dup = false;
#pragma unroll
            for (int p = 0; p < TAB_PROBES; p++) {
                const unsigned long long old = atomicCAS(&tab[h], TAB_EMPTY, v);
                if (old == TAB_EMPTY) { fresh++; break; }
                if (old == v) { dup = true; break; }
                h = (h + 1) & (TAB_SLOTS - 1);
            }
            if (!dup) {                   // first sighting in this workgroup (or the set was crowded)
                const uint64_t bit = 1ull << (v & 63);
                unsigned long long* word = reinterpret_cast<unsigned long long*>(bitmap) + (v >> 6);
                if (!(*word & bit)) atomicOr(word, (unsigned long long)bit);
            }
        }
        if (fresh) atomicAdd(&fresh_total, fresh);
        __syncthreads();
        const bool crowded = fresh_total > (uint32_t)(TAB_SLOTS * 3 / 4);
        __syncthreads();
        if (crowded) {                    // start over with an empty set; the bitmap keeps the truth
            for (int i = threadIdx.x; i < TAB_SLOTS; i += DD_THREADS) tab[i] = TAB_EMPTY;
            if (threadIdx.x == 0) fresh_total = 0;
            __syncthreads();
        }
    }
    if (bad) atomicCAS(&ctl->error, 0u, 3u /* -GIDS_E_RANGE */);
}

__global__ __launch_bounds__(DD_THREADS) void count_kernel(const uint64_t* __restrict__ bitmap, uint64_t n_words,
                                                           uint32_t* blocksum, uint32_t* blockoff, Ctl* ctl,
                                                           uint32_t* n_out) {
    __shared__ uint32_t smem[8];
    __shared__ uint32_t is_last;
    __shared__ uint32_t running;
    const uint64_t w0 = (uint64_t)blockIdx.x * WORDS_PER_BLOCK + (uint64_t)threadIdx.x * WORDS_PER_THREAD;
    uint32_t c = 0;
#pragma unroll
    for (int k = 0; k < WORDS_PER_THREAD; k++)
        if (w0 + k < n_words) c += __popcll(bitmap[w0 + k]);
    uint32_t total;
    block_exclusive_scan(c, &total, smem);
    if (threadIdx.x == 0) {
        __hip_atomic_store(&blocksum[blockIdx.x], total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __threadfence();
        const uint32_t tk = atomicAdd(&ctl->ticket, 1u);
        is_last = (tk == gridDim.x - 1);
        running = 0;
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();
    const uint32_t nb = gridDim.x;
    for (uint32_t base = 0; base < nb; base += DD_THREADS) {
        const uint32_t i = base + threadIdx.x;
        const uint32_t x = i < nb ? __hip_atomic_load(&blocksum[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
        uint32_t chunk;
        const uint32_t excl = block_exclusive_scan(x, &chunk, smem);
        if (i < nb) blockoff[i] = running + excl;
        __syncthreads();
        if (threadIdx.x == 0) running += chunk;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        *n_out = running;
        ctl->ticket = 0;
    }
}

// n_out_solo != nullptr: the bitmap fits one block, no count kernel ran; this block's total is the distinct count.
template <typename IdT>
__global__ __launch_bounds__(DD_THREADS) void emit_kernel(uint64_t* __restrict__ bitmap, uint64_t n_words,
                                                          const uint32_t* __restrict__ blockoff,
                                                          IdT* __restrict__ dst, uint8_t* __restrict__ reuse_inc,
                                                          uint32_t* __restrict__ wrank, int clear, const Ctl* ctl,
                                                          uint32_t* __restrict__ n_out_solo) {
    __shared__ uint32_t smem[8];
    const bool ok = ctl->error == 0;
    const uint64_t w0 = (uint64_t)blockIdx.x * WORDS_PER_BLOCK + (uint64_t)threadIdx.x * WORDS_PER_THREAD;
    uint64_t w[WORDS_PER_THREAD];
    uint32_t c = 0;
#pragma unroll
    for (int k = 0; k < WORDS_PER_THREAD; k++) {
        w[k] = (w0 + k < n_words) ? bitmap[w0 + k] : 0ull;
        c += __popcll(w[k]);
    }
    uint32_t total;
    uint32_t pos = block_exclusive_scan(c, &total, smem);
    if (n_out_solo) {
        if (threadIdx.x == 0) *n_out_solo = total;
    } else {
        pos += blockoff[blockIdx.x];
    }
#pragma unroll
    for (int k = 0; k < WORDS_PER_THREAD; k++) {
        uint64_t x = w[k];
        if (!x) continue;
        if (wrank) wrank[w0 + k] = pos;
        {
            // The list is written even when an error is pending (only valid IDs ever set a bit, and dst holds
            // every distinct ID of the raw list): the kernels that clear a kept bitmap find its words through
            // it.  What a failed operation must not change is the future-reuse counters.
            // Four set bits at a time: their counter updates are independent (the IDs are distinct, no two
            // threads share a byte), so the four loads go out together instead of one round trip per ID
            while (x) {
                uint64_t v[4];
                uint8_t r[4];
                int m = 0;
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    if (x) {
                        v[u] = (w0 + k) * 64 + (uint64_t)(__ffsll((unsigned long long)x) - 1);
                        x &= x - 1;
                        m = u + 1;
                    }
                }
                if (reuse_inc && ok) {
#pragma unroll
                    for (int u = 0; u < 4; u++)
                        if (u < m) r[u] = reuse_inc[v[u]];
#pragma unroll
                    for (int u = 0; u < 4; u++)
                        if (u < m) reuse_inc[v[u]] = (uint8_t)(r[u] + 1);
                }
#pragma unroll
                for (int u = 0; u < 4; u++)
                    if (u < m) dst[pos++] = (IdT)v[u];
            }
        }
        if (clear) bitmap[w0 + k] = 0ull;
    }
}

template <typename IdT>
__global__ void verify_kernel(const IdT* __restrict__ fresh, const IdT* __restrict__ head,
                              const uint32_t* __restrict__ head_n, Ctl* ctl) {
    if (ctl->error) return;
    const uint32_t n_u = ctl->n_unique, n_h = *head_n;
    bool bad = (n_u != n_h);
    const uint32_t m = n_u < n_h ? n_u : n_h;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < m; i += (uint64_t)gridDim.x * blockDim.x)
        if (fresh[i] != head[i]) bad = true;
    if (bad) atomicCAS(&ctl->error, 0u, 4u /* -GIDS_E_ORDER */);
}

template <typename IdT>
__global__ void inverse_kernel(const IdT* __restrict__ ids, uint64_t n, const uint64_t* __restrict__ bitmap,
                               const uint32_t* __restrict__ wrank, uint32_t* __restrict__ inverse, const Ctl* ctl) {
    if (ctl->error) return;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x) {
        const uint64_t v = (uint64_t)ids[i];
        const uint64_t word = bitmap[v >> 6];
        inverse[i] = wrank[v >> 6] + (uint32_t)__popcll(word & ((1ull << (v & 63)) - 1));
    }
}

template <typename IdT>
__global__ void clear_kernel(uint64_t* __restrict__ bitmap, const IdT* __restrict__ unique,
                             const uint32_t* __restrict__ n_u) {
    const uint32_t m = *n_u;
    for (uint64_t j = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; j < m; j += (uint64_t)gridDim.x * blockDim.x)
        bitmap[(uint64_t)unique[j] >> 6] = 0ull;
}

__global__ void fill_u32_kernel(uint32_t* p, uint64_t n, uint32_t value) {
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
        p[i] = value;
}
__global__ void fill_i64_kernel(int64_t* p, uint64_t n, int64_t value) {
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
        p[i] = value;
}

inline uint32_t blocks_for(uint64_t items, uint64_t per_block, uint32_t cap) {
    uint64_t b = (items + per_block - 1) / per_block;
    if (b < 1) b = 1;
    return (uint32_t)(b > cap ? cap : b);
}

}  // namespace

uint32_t scan_blocks(uint64_t n_words) { return (uint32_t)((n_words + WORDS_PER_BLOCK - 1) / WORDS_PER_BLOCK); }

template <typename IdT>
void launch_mark(const IdT* ids, uint64_t n, const uint32_t* n_dev, uint64_t n_rows, uint64_t* bitmap, Ctl* ctl,
                 hipStream_t s) {
    if (n == 0) return;
    const uint32_t grid = blocks_for(n, (uint64_t)DD_THREADS * MARK_ITEMS, 2048);
    hipLaunchKernelGGL(mark_kernel<IdT>, dim3(grid), dim3(DD_THREADS), 0, s, ids, n, n_dev, n_rows, bitmap, ctl);
}

void launch_count(const uint64_t* bitmap, uint64_t n_words, uint32_t* blocksum, uint32_t* blockoff, Ctl* ctl,
                  uint32_t* n_out, hipStream_t s) {
    hipLaunchKernelGGL(count_kernel, dim3(scan_blocks(n_words)), dim3(DD_THREADS), 0, s, bitmap, n_words, blocksum,
                       blockoff, ctl, n_out);
}

template <typename IdT>
void launch_emit(uint64_t* bitmap, uint64_t n_words, uint64_t, const uint32_t* blockoff, IdT* dst,
                 uint8_t* reuse_inc, uint32_t* wrank, bool clear, Ctl* ctl, uint32_t* n_out_solo, hipStream_t s) {
    hipLaunchKernelGGL(emit_kernel<IdT>, dim3(scan_blocks(n_words)), dim3(DD_THREADS), 0, s, bitmap, n_words,
                       blockoff, dst, reuse_inc, wrank, clear ? 1 : 0, ctl, n_out_solo);
}

template <typename IdT>
void launch_verify(const IdT* fresh, const IdT* head, const uint32_t* head_n, Ctl* ctl, uint64_t n_upper,
                   hipStream_t s) {
    hipLaunchKernelGGL(verify_kernel<IdT>, dim3(blocks_for(n_upper, 1024, 1024)), dim3(256), 0, s, fresh, head,
                       head_n, ctl);
}

template <typename IdT>
void launch_inverse(const IdT* ids, uint64_t n, const uint64_t* bitmap, const uint32_t* wrank, uint32_t* inverse,
                    Ctl* ctl, hipStream_t s) {
    if (n == 0) return;
    hipLaunchKernelGGL(inverse_kernel<IdT>, dim3(blocks_for(n, 1024, 2048)), dim3(256), 0, s, ids, n, bitmap, wrank,
                       inverse, ctl);
}

template <typename IdT>
void launch_clear(uint64_t* bitmap, const IdT* unique, const uint32_t* n_u, uint64_t n_upper, hipStream_t s) {
    hipLaunchKernelGGL(clear_kernel<IdT>, dim3(blocks_for(n_upper, 1024, 2048)), dim3(256), 0, s, bitmap, unique,
                       n_u);
}

void launch_fill_u32(uint32_t* p, uint64_t n, uint32_t value, hipStream_t s) {
    if (n == 0) return;
    hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks_for(n, 1024, 4096)), dim3(256), 0, s, p, n, value);
}
void launch_fill_i64(int64_t* p, uint64_t n, int64_t value, hipStream_t s) {
    if (n == 0) return;
    hipLaunchKernelGGL(fill_i64_kernel, dim3(blocks_for(n, 1024, 4096)), dim3(256), 0, s, p, n, value);
}

#define GIDS_INSTANTIATE(IdT)                                                                                      \
    template void launch_mark<IdT>(const IdT*, uint64_t, const uint32_t*, uint64_t, uint64_t*, Ctl*, hipStream_t); \
    template void launch_emit<IdT>(uint64_t*, uint64_t, uint64_t, const uint32_t*, IdT*, uint8_t*, uint32_t*, bool, \
                                   Ctl*, uint32_t*, hipStream_t);                                                  \
    template void launch_verify<IdT>(const IdT*, const IdT*, const uint32_t*, Ctl*, uint64_t, hipStream_t);        \
    template void launch_inverse<IdT>(const IdT*, uint64_t, const uint64_t*, const uint32_t*, uint32_t*, Ctl*,     \
                                      hipStream_t);                                                                \
    template void launch_clear<IdT>(uint64_t*, const IdT*, const uint32_t*, uint64_t, hipStream_t);
GIDS_INSTANTIATE(int32_t)
GIDS_INSTANTIATE(int64_t)

}  // namespace gids
