// Set-associative tag probe and victim selection of the GPU software cache
// with window buffering (GIDS paper, Section 3.4; CPU-buffer redirection,
// Section 3.3).
//
// The policy is batch-synchronous, so no lock is ever taken:
//   probe   every distinct ID of the minibatch is classified against the cache
//           state at the start of the minibatch.  `ways` adjacent lanes of a
//           wavefront compare one set's tags in one coalesced load and a ballot
//           names the matching way.  Hits stamp their line with the minibatch
//           index; misses set one bit (set, id / n_sets) in a per-set miss
//           mask.  The probe also takes this
//           minibatch's own entry out of the per-node future-reuse counters
//           (a reuse consumes one count, Section 3.4).
//   victim  a miss's rank among the misses of its set is a popcount of the
//           mask below its own bit (ascending ID order without any sort); the
//           lanes of its group rank the set's evictable ways by (stamp, way)
//           with cross-lane permutes, and the rank-th evictable way is its
//           victim.  A way is evictable when this minibatch did not touch it
//           and it is empty or its node's future-reuse counter is zero ("safe
//           to evict"); a positive counter is the "USE" state.  With more
//           misses than evictable ways the rest bypass the cache.
//   commit  writes the tag and stamp of every line a miss was given and clears
//           the miss mask; only then is the cache's metadata that of the next
//           minibatch's start.  The bytes follow in the row mover.
#include <cstdlib>

#include "gids_dev.h"

namespace gids {

namespace {

constexpr int CT_THREADS = 256;

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63; }

// bits of a 64-lane ballot that belong to this lane's group of `ways` lanes
__device__ __forceinline__ uint64_t group_bits(uint64_t ballot, uint32_t ways) {
    const uint32_t base = lane_id() & ~(ways - 1);
    const uint64_t mask = ways == 64 ? ~0ull : ((1ull << ways) - 1);
    return (ballot >> base) & mask;
}

template <typename IdT>
__global__ __launch_bounds__(CT_THREADS) void probe_kernel(CacheView<IdT> c, const IdT* __restrict__ unique,
                                                           const uint32_t* __restrict__ n_u_ptr, uint64_t out_capacity,
                                                           int pop_window, uint64_t* __restrict__ plan) {
    __shared__ uint32_t block_cnt[3];
    Ctl* ctl = c.ctl;
    if (ctl->error) return;                                  // set only by earlier kernels: uniform
    const uint32_t n_u = *n_u_ptr;
    if (n_u > out_capacity) {                                // the same verdict in every thread
        if (blockIdx.x == 0 && threadIdx.x == 0) ctl->error = 7u; /* -GIDS_E_SPACE; finalize reports it */
        return;
    }
    if (threadIdx.x < 3) block_cnt[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t ways = c.ways, lg = c.lg_ways;
    const uint32_t per_wave = 64u >> lg;                     // IDs a wavefront classifies at once
    const uint32_t sub = lane_id() & (ways - 1);             // this lane's way
    const bool leader = sub == 0;
    const uint32_t stamp = ctl->stamp;
    const uint64_t wave0 = ((uint64_t)blockIdx.x * CT_THREADS + threadIdx.x) >> 6;
    const uint64_t n_waves = ((uint64_t)gridDim.x * CT_THREADS) >> 6;
    uint32_t hits = 0, cpus = 0, misses = 0;
    for (uint64_t chunk = wave0; chunk * per_wave < n_u; chunk += n_waves) {
        const uint64_t j = chunk * per_wave + (lane_id() >> lg);
        const bool valid = j < n_u;
        const uint64_t v = valid ? (uint64_t)unique[j] : 0;
        // leader: CPU-buffer membership, window pop
        uint32_t hot = 0, slot = 0;
        if (valid && leader) {
            if (pop_window) c.reuse[v] = (uint8_t)(c.reuse[v] - 1);
            if (c.hotbits) {
                const uint64_t hw = c.hotbits[v >> 6];
                const uint64_t bit = 1ull << (v & 63);
                if (hw & bit) {
                    hot = 1;
                    slot = c.hotrank[v >> 6] + (uint32_t)__popcll(hw & (bit - 1));
                }
            }
        }
        hot = __shfl(hot, (int)(lane_id() & ~(ways - 1)));
        const uint64_t b = store_line_of(c, v);              // the tag: v itself with one row per line
        uint64_t set = 0, round = 0;
        set_and_round(c, b, &set, &round);
        bool match = false;
        if (valid && !hot) match = (uint64_t)c.tags[set * ways + sub] == b;   // empty lines hold -1
        const uint64_t gb = group_bits(__ballot(match), ways);
        const bool is_hit = gb != 0;
        if (valid && leader) {
            if (hot) {
                plan[j] = (PLAN_CPU << PLAN_SHIFT) | slot;
                cpus++;
            } else if (is_hit) {
                const uint64_t line = set * ways + (uint32_t)(__ffsll((unsigned long long)gb) - 1);
                c.stamps[line] = (int32_t)stamp;
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
    // one global atomic per block and counter (same-address atomics serialise in L2)
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        hits += __shfl_down(hits, d);
        cpus += __shfl_down(cpus, d);
        misses += __shfl_down(misses, d);
    }
    if (lane_id() == 0) {
        if (hits) atomicAdd(&block_cnt[0], hits);
        if (cpus) atomicAdd(&block_cnt[1], cpus);
        if (misses) atomicAdd(&block_cnt[2], misses);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (block_cnt[0]) atomicAdd(&ctl->cnt_hit, block_cnt[0]);
        if (block_cnt[1]) atomicAdd(&ctl->cnt_cpu, block_cnt[1]);
        if (block_cnt[2]) atomicAdd(&ctl->cnt_miss, block_cnt[2]);
    }
}

template <typename IdT>
__global__ __launch_bounds__(CT_THREADS) void victim_kernel(CacheView<IdT> c, const IdT* __restrict__ unique,
                                                            const uint32_t* __restrict__ n_u_ptr,
                                                            uint64_t* __restrict__ plan) {
    __shared__ uint32_t block_byp, block_fill;
    Ctl* ctl = c.ctl;
    if (ctl->error || ctl->cnt_miss == 0) return;            // cnt_miss is final: the probe has ended
    if (threadIdx.x == 0) block_byp = block_fill = 0;
    __syncthreads();
    const uint32_t n_u = *n_u_ptr;
    const uint32_t ways = c.ways, lg = c.lg_ways;
    const uint32_t per_wave = 64u >> lg;
    const uint32_t sub = lane_id() & (ways - 1);
    const uint32_t group_base = lane_id() & ~(ways - 1);
    const int32_t stamp = (int32_t)ctl->stamp;
    const uint64_t wave0 = ((uint64_t)blockIdx.x * CT_THREADS + threadIdx.x) >> 6;
    const uint64_t n_waves = ((uint64_t)gridDim.x * CT_THREADS) >> 6;
    const uint64_t rpl = c.rows_per_line;
    uint32_t bypasses = 0, fills = 0;
    for (uint64_t chunk = wave0; chunk * per_wave < n_u; chunk += n_waves) {
        const uint64_t j = chunk * per_wave + (lane_id() >> lg);
        const bool valid = j < n_u && (plan[j] >> PLAN_SHIFT) == PLAN_MISS_TBD;
        if (!__ballot(valid)) continue;                      // no miss among this wave's IDs
        const uint64_t v = valid ? (uint64_t)unique[j] : 0;
        const uint64_t b = store_line_of(c, v);
        uint64_t set = 0, round = 0;
        set_and_round(c, b, &set, &round);
        // this lane's way: evictable?
        const uint64_t line = set * ways + sub;
        bool ev = false, empty = false;
        int32_t st = 0;
        if (valid) {
            const IdT tg = c.tags[line];
            st = c.stamps[line];
            empty = tg < 0;
            bool pinned = false;                             // some row of the line has a buffered future use
            if (!empty) {
                if (rpl == 1) {
                    pinned = c.reuse[(uint64_t)tg] != 0;
                } else {
                    const uint64_t r0 = (uint64_t)tg * rpl;
                    const uint64_t r1 = r0 + rpl < c.n_rows ? r0 + rpl : c.n_rows;
                    for (uint64_t r = r0; r < r1; r++) pinned |= c.reuse[r] != 0;
                }
            }
            ev = st != stamp && !pinned;
        }
        // order of this way among the set's evictable ways: by (stamp, way), empty ways (stamp -1) first;
        // under the random base policy occupied ways are ordered by a hash of (minibatch, set, way) instead
        uint64_t order = (uint64_t)(uint32_t)(st + 1);
        if (c.policy == 1)
            order = empty ? 0ull : 1ull + (mix64(mix64(mix64(c.policy_key ^ (uint64_t)(uint32_t)stamp) ^ set) ^ sub) >> 9);
        const uint64_t key = ev ? (order << 8) | sub : ~0ull;
        uint32_t way_rank = 0;
        for (uint32_t o = 0; o < ways; o++) {
            const uint64_t other = __shfl(key, (int)(group_base + o));
            way_rank += other < key;
        }
        const uint32_t n_ev = (uint32_t)__popcll(group_bits(__ballot(ev), ways));
        // rank of this miss among its set's misses in ascending ID order
        uint32_t k = 0;
        if (valid && sub == 0) {
            const uint64_t* m = c.missmask + set * c.words_per_set;
            const uint32_t wi = (uint32_t)(round >> 6);
            for (uint32_t x = 0; x < wi; x++) k += (uint32_t)__popcll(m[x]);
            k += (uint32_t)__popcll(m[wi] & ((1ull << (round & 63)) - 1));
        }
        k = __shfl(k, (int)group_base);
        // With several rows per line the IDs of one missing line sit next to each other in the ascending list
        // and all find the same way; the first of them that is not served by the CPU buffer fills the line,
        // the others only fetch their own row.  (Kinds other than CPU are misses here: the line is absent.)
        uint32_t follow = 0;
        if (valid && sub == 0 && rpl > 1) {
            for (uint64_t i = j; i-- > 0;) {
                if (store_line_of(c, (uint64_t)unique[i]) != b) break;
                if ((plan[i] >> PLAN_SHIFT) != PLAN_CPU) { follow = 1; break; }
            }
        }
        follow = __shfl(follow, (int)group_base);
        if (valid) {
            if (ev && way_rank == k) plan[j] = ((follow ? PLAN_FOLLOW : PLAN_INSTALL) << PLAN_SHIFT) | line;
            if (sub == 0) {
                if (k >= n_ev) {
                    plan[j] = PLAN_BYPASS << PLAN_SHIFT;
                    bypasses++;
                } else if (!follow) {
                    fills++;
                }
            }
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        bypasses += __shfl_down(bypasses, d);
        fills += __shfl_down(fills, d);
    }
    if (lane_id() == 0 && bypasses) atomicAdd(&block_byp, bypasses);
    if (lane_id() == 0 && fills) atomicAdd(&block_fill, fills);
    __syncthreads();
    if (threadIdx.x == 0 && block_byp) atomicAdd(&ctl->cnt_bypass, block_byp);
    if (threadIdx.x == 0 && block_fill) atomicAdd(&ctl->cnt_fill, block_fill);
}

// Publishes the gather's decisions: tag and stamp of every line a miss will
// fill, the miss mask back to zero, and the header the row mover reads.  After
// this kernel the next minibatch may be classified, whether or not the rows of
// this one have moved yet.
template <typename IdT>
__global__ __launch_bounds__(CT_THREADS) void commit_kernel(CacheView<IdT> c, const IdT* __restrict__ unique,
                                                            const uint32_t* __restrict__ n_u_ptr,
                                                            const uint64_t* __restrict__ plan, BatchHdr* hdr) {
    const Ctl* ctl = c.ctl;
    const bool ok = ctl->error == 0;
    const uint32_t n_u = ok ? *n_u_ptr : 0;
    const uint32_t stamp = ctl->stamp;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        hdr->ok = ok ? 1u : 0u;
        hdr->n_u = n_u;
        hdr->stamp = stamp;
        hdr->next_chunk = 0;
    }
    if (!ok || ctl->cnt_miss == 0) return;
    for (uint64_t j = (uint64_t)blockIdx.x * CT_THREADS + threadIdx.x; j < n_u; j += (uint64_t)gridDim.x * CT_THREADS) {
        const uint64_t e = plan[j];
        const uint64_t kind = e >> PLAN_SHIFT;
        if (kind < PLAN_INSTALL) continue;
        const uint64_t b = store_line_of(c, (uint64_t)unique[j]);
        if (kind == PLAN_INSTALL) {
            const uint64_t line = e & PLAN_INDEX_MASK;
            c.tags[line] = (IdT)b;
            c.stamps[line] = (int32_t)stamp;
        }
        uint64_t set, round;
        set_and_round(c, b, &set, &round);
        c.missmask[set * c.words_per_set + (round >> 6)] = 0ull;
    }
}

inline uint32_t probe_cap() {
    static const uint32_t cap = [] {
        const char* e = getenv("GIDS_PROBE_BLOCKS");
        const int v = e ? atoi(e) : 2048;
        return (uint32_t)(v >= 1 && v <= 65536 ? v : 2048);
    }();
    return cap;
}

inline uint32_t grid_for(uint64_t groups, uint32_t ways, uint32_t cap) {
    const uint64_t per_block = (uint64_t)(CT_THREADS / 64) * (64 / ways);
    uint64_t b = (groups + per_block - 1) / per_block;
    if (b < 1) b = 1;
    return (uint32_t)(b > cap ? cap : b);
}

}  // namespace

template <typename IdT>
void launch_probe(const CacheView<IdT>& c, const IdT* unique, const uint32_t* n_u, uint64_t n_upper,
                  uint64_t out_capacity, bool pop_window, uint64_t* plan, hipStream_t s) {
    hipLaunchKernelGGL(probe_kernel<IdT>, dim3(grid_for(n_upper, c.ways, probe_cap())), dim3(CT_THREADS), 0, s, c, unique,
                       n_u, out_capacity, pop_window ? 1 : 0, plan);
}

template <typename IdT>
void launch_commit(const CacheView<IdT>& c, const IdT* unique, const uint32_t* n_u, uint64_t n_upper,
                   const uint64_t* plan, BatchHdr* hdr, hipStream_t s) {
    uint64_t b = (n_upper + CT_THREADS - 1) / CT_THREADS;
    if (b < 1) b = 1;
    if (b > 1024) b = 1024;
    hipLaunchKernelGGL(commit_kernel<IdT>, dim3((uint32_t)b), dim3(CT_THREADS), 0, s, c, unique, n_u, plan, hdr);
}

template <typename IdT>
void launch_victim(const CacheView<IdT>& c, const IdT* unique, const uint32_t* n_u, uint64_t n_upper,
                   uint64_t* plan, hipStream_t s) {
    hipLaunchKernelGGL(victim_kernel<IdT>, dim3(grid_for(n_upper, c.ways, probe_cap())), dim3(CT_THREADS), 0, s, c, unique,
                       n_u, plan);
}

#define GIDS_INSTANTIATE(IdT)                                                                                       \
    template void launch_probe<IdT>(const CacheView<IdT>&, const IdT*, const uint32_t*, uint64_t, uint64_t, bool,   \
                                    uint64_t*, hipStream_t);                                                        \
    template void launch_commit<IdT>(const CacheView<IdT>&, const IdT*, const uint32_t*, uint64_t, const uint64_t*, \
                                     BatchHdr*, hipStream_t);                                                       \
    template void launch_victim<IdT>(const CacheView<IdT>&, const IdT*, const uint32_t*, uint64_t, uint64_t*,       \
                                     hipStream_t);
GIDS_INSTANTIATE(int32_t)
GIDS_INSTANTIATE(int64_t)

}  // namespace gids
