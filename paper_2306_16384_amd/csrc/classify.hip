// Fused classification of one minibatch for short ID lists: CPU-buffer lookup,
// tag probe, victim selection, publication of tags and stamps, the
// accumulator's queueing and the counters in ONE launch (GIDS paper: cache with
// window buffering, Section 3.4; CPU-buffer redirection, Section 3.3;
// accumulator, Section 3.2).
//
// The separate probe / victim / commit / queue / finalize kernels need a launch
// boundary between them because a set's ways are ranked only after every ID of
// the minibatch has been probed.  That dependency never crosses a cache set, so
// here the sets are dealt out to the workgroups (set s belongs to workgroup
// s mod gridDim.x): every workgroup scans the whole distinct-ID list, keeps the
// IDs of its own sets, and takes them through all phases with nothing but
// workgroup barriers in between.  One thread per ID; the `ways` tags of a set
// are read by that thread (ways <= 16).  The last workgroup to finish publishes
// the counters.  A minibatch that takes one launch instead of five matters when
// the launches themselves are the cost: short lists, and lists classified
// beside a row mover that saturates the host link.
#include "gather_dev.h"
#include "gids_dev.h"

namespace gids {

namespace {

constexpr int CL_THREADS = 256;
constexpr int CL_UNROLL = 4;               // list entries a thread fetches before it looks at any

__device__ __forceinline__ uint32_t ld_agent(const uint32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// set s is classified by workgroup s mod n_wg
template <typename IdT>
__device__ __forceinline__ bool owns(const CacheView<IdT>& c, uint64_t set, uint32_t n_wg, uint32_t me) {
    return c.use32 ? (uint32_t)set % n_wg == me : set % n_wg == me;
}

template <typename IdT, int WAYS>
__global__ __launch_bounds__(CL_THREADS) void classify_kernel(CacheView<IdT> c, AccumView a, uint32_t group, int accum,
                                                              const IdT* __restrict__ unique,
                                                              const uint32_t* __restrict__ n_u_ptr,
                                                              uint64_t out_capacity, int pop_window,
                                                              uint64_t* __restrict__ plan, BatchHdr* hdr,
                                                              char* __restrict__ out, IdT* __restrict__ unique_out,
                                                              StatsRec* rec, uint64_t seq) {
    __shared__ uint32_t cnt[5];                              // hits, CPU-buffer hits, misses, bypasses, line fills
    __shared__ uint32_t is_last;
    Ctl* ctl = c.ctl;
    const uint32_t tid = threadIdx.x;
    const uint32_t n_u = *n_u_ptr;
    // the same verdict in every workgroup: an error left by an earlier kernel, or an output that is too small
    const bool too_many = n_u > out_capacity;
    const bool ok = ld_agent(&ctl->error) == 0 && !too_many;
    const int32_t stamp = (int32_t)ctl->stamp;
    const uint32_t n_wg = gridDim.x, me = blockIdx.x;
    if (tid < 5) cnt[tid] = 0;
    __syncthreads();
    uint32_t hits = 0, cpus = 0, misses = 0, bypasses = 0, fills = 0;
    if (ok) {
        // ---- probe: every ID of this workgroup's sets against the state at the start of the minibatch
        for (uint64_t base = tid; base < n_u; base += (uint64_t)CL_THREADS * CL_UNROLL) {
            uint64_t vv[CL_UNROLL];
#pragma unroll
            for (int u = 0; u < CL_UNROLL; u++) {
                const uint64_t j = base + (uint64_t)u * CL_THREADS;
                vv[u] = j < n_u ? (uint64_t)unique[j] : ~0ull;
            }
#pragma unroll
            for (int u = 0; u < CL_UNROLL; u++) {
                const uint64_t j = base + (uint64_t)u * CL_THREADS;
                const uint64_t v = vv[u];
                if (v == ~0ull) continue;
                uint64_t set, round;
                set_and_round(c, v, &set, &round);
                if (!owns(c, set, n_wg, me)) continue;
                if (pop_window) c.reuse[v] = (uint8_t)(c.reuse[v] - 1);
                if (c.hotbits) {
                    const uint64_t hw = c.hotbits[v >> 6];
                    const uint64_t bit = 1ull << (v & 63);
                    if (hw & bit) {
                        plan[j] = (PLAN_CPU << PLAN_SHIFT) | (c.hotrank[v >> 6] + (uint32_t)__popcll(hw & (bit - 1)));
                        cpus++;
                        continue;
                    }
                }
                const IdT* row = c.tags + set * WAYS;
                int way = -1;
#pragma unroll
                for (int w = 0; w < WAYS; w++)
                    if ((uint64_t)row[w] == v) way = w;          // empty lines hold -1
                if (way >= 0) {
                    const uint64_t line = set * WAYS + (uint32_t)way;
                    c.stamps[line] = stamp;
                    plan[j] = (PLAN_HIT << PLAN_SHIFT) | line;
                    hits++;
                } else {
                    plan[j] = PLAN_MISS_TBD << PLAN_SHIFT;
                    atomicOr(reinterpret_cast<unsigned long long*>(c.missmask) + set * c.words_per_set + (round >> 6),
                             1ull << (round & 63));
                    misses++;
                }
            }
        }
        if (misses) atomicAdd(&cnt[2], misses);
        __threadfence();
        __syncthreads();
        // ---- victims: the k-th miss of a set (ascending ID) takes the k-th evictable way in (stamp, way) order
        if (cnt[2]) {
            for (uint64_t base = tid; base < n_u; base += (uint64_t)CL_THREADS * CL_UNROLL) {
                uint64_t ee[CL_UNROLL];
#pragma unroll
                for (int u = 0; u < CL_UNROLL; u++) {
                    const uint64_t j = base + (uint64_t)u * CL_THREADS;
                    ee[u] = j < n_u ? plan[j] : 0ull;             // entries of other workgroups' sets are skipped below
                }
#pragma unroll
                for (int u = 0; u < CL_UNROLL; u++) {
                    const uint64_t j = base + (uint64_t)u * CL_THREADS;
                    if (j >= n_u || (ee[u] >> PLAN_SHIFT) != PLAN_MISS_TBD) continue;
                    const uint64_t v = (uint64_t)unique[j];
                    uint64_t set, round;
                    set_and_round(c, v, &set, &round);
                    if (!owns(c, set, n_wg, me)) continue;        // (a stale entry of an earlier minibatch)
                    const uint64_t line0 = set * WAYS;
                    IdT tg[WAYS];
                    int32_t st[WAYS];
#pragma unroll
                    for (int w = 0; w < WAYS; w++) {
                        tg[w] = c.tags[line0 + w];
                        st[w] = c.stamps[line0 + w];
                    }
                    uint8_t ru[WAYS];
#pragma unroll
                    for (int w = 0; w < WAYS; w++) ru[w] = tg[w] < 0 ? (uint8_t)0 : c.reuse[(uint64_t)tg[w]];
                    uint64_t key[WAYS];
                    uint32_t n_ev = 0;
#pragma unroll
                    for (int w = 0; w < WAYS; w++) {
                        const bool empty = tg[w] < 0;
                        const bool ev = st[w] != stamp && ru[w] == 0;   // untouched in this minibatch, no buffered future use
                        uint64_t order = (uint64_t)(uint32_t)(st[w] + 1);
                        if (c.policy == 1)
                            order = empty ? 0ull
                                          : 1ull + (mix64(mix64(mix64(c.policy_key ^ (uint64_t)(uint32_t)stamp) ^ set) ^ (uint64_t)w) >> 9);
                        key[w] = ev ? (order << 8) | (uint64_t)w : ~0ull;
                        n_ev += ev;
                    }
                    // rank of this miss among its set's misses in ascending ID order
                    uint32_t k = 0;
                    const uint64_t* m = c.missmask + set * c.words_per_set;
                    const uint32_t wi = (uint32_t)(round >> 6);
                    for (uint32_t x = 0; x < wi; x++) k += (uint32_t)__popcll(m[x]);
                    k += (uint32_t)__popcll(m[wi] & ((1ull << (round & 63)) - 1));
                    if (k >= n_ev) {
                        plan[j] = PLAN_BYPASS << PLAN_SHIFT;
                        bypasses++;
                    } else {
                        int way = 0;
#pragma unroll
                        for (int w = 0; w < WAYS; w++) {
                            uint32_t r = 0;
#pragma unroll
                            for (int o = 0; o < WAYS; o++) r += key[o] < key[w];
                            if (key[w] != ~0ull && r == k) way = w;
                        }
                        plan[j] = (PLAN_INSTALL << PLAN_SHIFT) | (line0 + (uint32_t)way);
                        fills++;
                    }
                }
            }
            __threadfence();
            __syncthreads();
        }
        // ---- publish tags and stamps, clear the miss mask; with the accumulator, queue every row
        if (cnt[2] || accum) {
            for (uint64_t base = 0; base < n_u; base += CL_THREADS) {    // uniform trip count: queue_entry ballots
                const uint64_t j = base + tid;
                bool mine = false;
                uint64_t e = 0, v = 0;
                if (j < n_u) {
                    v = (uint64_t)unique[j];
                    uint64_t set, round;
                    set_and_round(c, v, &set, &round);
                    mine = owns(c, set, n_wg, me);
                    if (mine) {
                        e = plan[j];
                        const uint64_t kind = e >> PLAN_SHIFT;
                        if (kind >= PLAN_INSTALL) {
                            if (kind == PLAN_INSTALL) {
                                const uint64_t line = e & PLAN_INDEX_MASK;
                                c.tags[line] = (IdT)v;
                                c.stamps[line] = stamp;
                            }
                            c.missmask[set * c.words_per_set + (round >> 6)] = 0ull;
                        }
                    }
                }
                if (accum) queue_entry(c, a, group, mine, j, e, v, out, unique_out);
            }
        }
    }
    // ---- counters; the last workgroup to get here publishes them and the header the row mover reads
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        hits += __shfl_down(hits, d);
        cpus += __shfl_down(cpus, d);
        bypasses += __shfl_down(bypasses, d);
        fills += __shfl_down(fills, d);
    }
    if ((tid & 63) == 0) {
        if (hits) atomicAdd(&cnt[0], hits);
        if (cpus) atomicAdd(&cnt[1], cpus);
        if (bypasses) atomicAdd(&cnt[3], bypasses);
        if (fills) atomicAdd(&cnt[4], fills);
    }
    __syncthreads();
    if (tid == 0) {
        if (cnt[0]) atomicAdd(&ctl->cnt_hit, cnt[0]);
        if (cnt[1]) atomicAdd(&ctl->cnt_cpu, cnt[1]);
        if (cnt[2]) atomicAdd(&ctl->cnt_miss, cnt[2]);
        if (cnt[3]) atomicAdd(&ctl->cnt_bypass, cnt[3]);
        if (cnt[4]) atomicAdd(&ctl->cnt_fill, cnt[4]);
        __threadfence();
        is_last = atomicAdd(&ctl->ticket_cls, 1u) == n_wg - 1;
    }
    __syncthreads();
    if (!is_last || tid != 0) return;
    __threadfence();
    if (too_many) atomicCAS(&ctl->error, 0u, 7u /* -GIDS_E_SPACE */);
    const bool good = ld_agent(&ctl->error) == 0;
    hdr->ok = good ? 1u : 0u;
    hdr->n_u = good ? n_u : 0u;
    hdr->stamp = (uint32_t)stamp;
    hdr->next_chunk = 0;
    ctl->ticket_cls = 0;
    publish_stats(ctl, rec, seq, n_u, accum);
}

}  // namespace

uint32_t classify_max_ways() { return 16; }

template <typename IdT>
void launch_classify(const CacheView<IdT>& c, const AccumView& a, uint32_t group, int accum, const IdT* unique,
                     const uint32_t* n_u, uint64_t n_upper, uint64_t out_capacity, bool pop_window, uint64_t* plan,
                     BatchHdr* hdr, char* out, IdT* unique_out, StatsRec* rec, uint64_t seq, hipStream_t s) {
    // about 128 list entries per workgroup's own share; every workgroup reads the whole list
    uint64_t g = (n_upper + 127) / 128;
    if (g < 1) g = 1;
    if (g > 128) g = 128;
    if (g > c.n_sets) g = c.n_sets;                          // a workgroup without a set would only take a ticket
#define GIDS_CLASSIFY(W)                                                                                          \
    hipLaunchKernelGGL((classify_kernel<IdT, W>), dim3((uint32_t)g), dim3(CL_THREADS), 0, s, c, a, group, accum,  \
                       unique, n_u, out_capacity, pop_window ? 1 : 0, plan, hdr, out, unique_out, rec, seq)
    switch (c.ways) {
        case 1: GIDS_CLASSIFY(1); break;
        case 2: GIDS_CLASSIFY(2); break;
        case 4: GIDS_CLASSIFY(4); break;
        case 8: GIDS_CLASSIFY(8); break;
        default: GIDS_CLASSIFY(16); break;
    }
#undef GIDS_CLASSIFY
}

#define GIDS_INSTANTIATE(IdT)                                                                                     \
    template void launch_classify<IdT>(const CacheView<IdT>&, const AccumView&, uint32_t, int, const IdT*,        \
                                       const uint32_t*, uint64_t, uint64_t, bool, uint64_t*, BatchHdr*, char*,    \
                                       IdT*, StatsRec*, uint64_t, hipStream_t);
GIDS_INSTANTIATE(int32_t)
GIDS_INSTANTIATE(int64_t)

}  // namespace gids
