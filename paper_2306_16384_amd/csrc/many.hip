// Merged iterations (GIDS paper, Section 3.2: the data preparation of several
// consecutive iterations is merged so that the stop-and-go boundaries between
// minibatches disappear).  One call brings k steps, each "push one future list,
// gather the window's head"; here all k steps run in two launches, whatever k,
// followed by the group mover's:
//
//   dedup_small   one workgroup per pushed list: the list is marked into a
//                 bitmap in LDS (tables whose bitmap fits a workgroup's LDS:
//                 1.3 M rows on gfx950; larger tables go through the
//                 per-list kernels and the bitmap in device memory), scanned
//                 and written out as ascending distinct IDs.  Nothing else
//                 of the push happens here.
//   classify_many the k steps one after the other inside one kernel.  A step's
//                 decisions depend only on the state of the cache sets its IDs
//                 fall into, and so does everything a step changes (tags,
//                 stamps, the future-reuse counters of the nodes that map to a
//                 set, the accumulator's words per line): the sets are dealt
//                 out to the workgroups (set s belongs to workgroup s mod
//                 gridDim.x, a power of two), and no workgroup waits for
//                 another.  A workgroup reads every list once and keeps the
//                 IDs of its own sets in LDS; where it fits, the state of its
//                 sets lives in LDS as well for the length of the kernel, and
//                 the steps then touch device memory only to store the
//                 group's operations.  Per step: the pushed list's
//                 future-reuse counters +1 (Section 3.4, Fig. 6); the head
//                 list's counters -1, CPU-buffer lookup (Section 3.3), tag
//                 probe; victims; commit and the accumulator's queueing (every
//                 row becomes an operation of the open group, whose mover runs
//                 after this kernel), with workgroup barriers between the
//                 phases.  One thread per ID, the `ways` tags of a set read by
//                 that thread (ways <= 16).  The last workgroup to finish
//                 publishes the k records of counters.
#include <cstdlib>

#include "gather_dev.h"
#include "gids_dev.h"

namespace gids {

namespace {

constexpr int DS_THREADS = 1024;
constexpr int CM_THREADS = 1024;
constexpr int CM_UNROLL = 4;               // list entries a thread fetches before it looks at any
constexpr int CM_SCAN = 8;                 // list entries a thread has in flight when it picks out its workgroup's
constexpr uint32_t CM_NONE = 0xFFFFFFFFu;  // not a CPU-buffer row
constexpr uint64_t MANY_LDS_MAX_BYTES = 152 * 1024;    // dynamic, of a CU's 160 KiB of LDS

template <typename IdT>
__global__ __launch_bounds__(DS_THREADS) void dedup_small_kernel(ManyPushes<IdT> p, uint64_t n_rows, Ctl* ctl) {
    extern __shared__ unsigned long long bm[];               // n_words words: the launcher sizes it for the table
    __shared__ uint32_t wave_sum[DS_THREADS / 64];
    const uint32_t tid = threadIdx.x;
    const IdT* __restrict__ ids = p.ids[blockIdx.x];
    const uint64_t n = p.n[blockIdx.x];
    IdT* __restrict__ dst = p.dst[blockIdx.x];
    const uint32_t n_words = (uint32_t)((n_rows + 63) / 64);
    for (uint32_t w = tid; w < n_words; w += DS_THREADS) bm[w] = 0ull;
    __syncthreads();
    bool bad = false;
    for (uint64_t i = tid; i < n; i += DS_THREADS) {
        const IdT raw = ids[i];
        if (raw < 0 || (uint64_t)raw >= n_rows) { bad = true; continue; }
        const uint64_t v = (uint64_t)raw;
        atomicOr(&bm[v >> 6], 1ull << (v & 63));
    }
    if (bad) atomicCAS(&ctl->error, 0u, 3u /* -GIDS_E_RANGE */);
    __syncthreads();
    // every thread takes a run of consecutive words: population count, workgroup prefix, then the bit positions
    const uint32_t per = (n_words + DS_THREADS - 1) / DS_THREADS;
    const uint32_t w0 = tid * per, w1 = w0 + per < n_words ? w0 + per : n_words;
    uint32_t c = 0;
    for (uint32_t w = w0; w < w1; w++) c += (uint32_t)__popcll(bm[w]);
    uint32_t incl = c;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = __shfl_up(incl, d);
        if ((tid & 63) >= (uint32_t)d) incl += y;
    }
    if ((tid & 63) == 63) wave_sum[tid >> 6] = incl;
    __syncthreads();
    uint32_t base = 0, total = 0;
#pragma unroll
    for (int w = 0; w < DS_THREADS / 64; w++) {
        const uint32_t s = wave_sum[w];
        if ((uint32_t)w < (tid >> 6)) base += s;
        total += s;
    }
    uint32_t pos = base + incl - c;
    for (uint32_t w = w0; w < w1; w++) {
        unsigned long long x = bm[w];
        while (x) {
            dst[pos++] = (IdT)((uint64_t)w * 64 + (uint64_t)(__ffsll(x) - 1));
            x &= x - 1;
        }
    }
    if (tid == 0) ctl->win_n[p.slot[blockIdx.x]] = total;
}

template <typename IdT>
__device__ __forceinline__ bool owns(const CacheView<IdT>& c, uint64_t set, uint32_t n_wg, uint32_t me) {
    return c.use32 ? (uint32_t)set % n_wg == me : set % n_wg == me;
}

// the list pushed in a step: one more buffered future use for each of its nodes that this workgroup owns
template <typename IdT>
__device__ __forceinline__ void raise_counters(const CacheView<IdT>& c, const IdT* __restrict__ P, uint32_t n_p,
                                               uint32_t n_wg, uint32_t me) {
    for (uint64_t base = threadIdx.x; base < n_p; base += (uint64_t)blockDim.x * CM_UNROLL) {
        uint64_t vv[CM_UNROLL];
#pragma unroll
        for (int u = 0; u < CM_UNROLL; u++) {
            const uint64_t j = base + (uint64_t)u * blockDim.x;
            vv[u] = j < n_p ? (uint64_t)P[j] : ~0ull;
        }
#pragma unroll
        for (int u = 0; u < CM_UNROLL; u++) {
            if (vv[u] == ~0ull) continue;
            uint64_t set, round;
            set_and_round(c, vv[u], &set, &round);
            if (owns(c, set, n_wg, me)) c.reuse[vv[u]] = (uint8_t)(c.reuse[vv[u]] + 1);
        }
    }
}

// Where the steps of a merged call find the state they read and write: the tags and stamps of a set's lines,
// its miss mask, the future-reuse counters of the nodes that map to it, and the words the accumulator keeps per
// line.  `slot` names a set in that place, `node` a node's counter.
//
// In device memory, where the per-step kernels keep it: a set by its number, a node by its ID.
template <typename IdT, int WAYS>
struct StateInMemory {
    static constexpr bool in_lds = false;
    const CacheView<IdT>& c;
    LineWordsGlobal lw;
    __device__ __forceinline__ uint32_t slot_of(uint32_t set, uint32_t) const { return set; }
    __device__ __forceinline__ uint32_t node_of(uint32_t, uint32_t, uint32_t v) const { return v; }
    __device__ __forceinline__ uint32_t node_of_tag(uint32_t, uint32_t tag) const { return tag; }
    __device__ __forceinline__ IdT* tags(uint32_t slot) const { return c.tags + (uint64_t)slot * WAYS; }
    __device__ __forceinline__ int32_t* stamps(uint32_t slot) const { return c.stamps + (uint64_t)slot * WAYS; }
    __device__ __forceinline__ uint8_t* counter(uint32_t node) const { return c.reuse + node; }
    __device__ __forceinline__ unsigned long long* miss_words(uint32_t slot) const {
        return reinterpret_cast<unsigned long long*>(c.missmask) + (uint64_t)slot * c.words_per_set;
    }
    __device__ __forceinline__ uint32_t local_line(uint32_t, int) const { return 0; }
    // the word that remembers the output row of the call's first fill of a CPU-buffer row (nullptr: not kept)
    __device__ __forceinline__ char** first_out(uint32_t cpu_row, uint32_t) const {
        return c.cpu_first ? c.cpu_first + cpu_row : nullptr;
    }
};

// The per-line words of the accumulator for the lines of this workgroup's sets, in LDS.  Deferred: an installed
// line's fill waits here (pend = its node, bit 31 = it fills the line late; pout = its output row) while
// fgrp is the call's group.
struct LineWordsLds {
    static constexpr bool deferred = true;
    uint32_t* pend;
    uint32_t* fgrp;
    uint32_t* hgrp;
    char** pout;
    __device__ __forceinline__ uint32_t fill_group(uint64_t, uint32_t local) const { return fgrp[local]; }
    __device__ __forceinline__ uint32_t hit_group(uint64_t, uint32_t local) const { return hgrp[local]; }
    __device__ __forceinline__ uint32_t pending_fill(uint64_t, uint32_t local) const { return pend[local]; }
    __device__ __forceinline__ void* pending_out(uint64_t, uint32_t local, uint32_t) const { return pout[local]; }
    __device__ __forceinline__ uint32_t waiting_node(uint32_t local) const { return pend[local] & 0x7FFFFFFFu; }
    __device__ __forceinline__ void wait_fill(uint32_t local, uint32_t group, uint32_t node, bool late, char* dst) const {
        fgrp[local] = group;
        pend[local] = node | (late ? 0x80000000u : 0u);
        pout[local] = dst;
    }
    __device__ __forceinline__ void note_fill(uint64_t, uint32_t, uint32_t, uint32_t, char*) const {}
    __device__ __forceinline__ void note_hit(uint64_t, uint32_t local, uint32_t group) const { hgrp[local] = group; }
};

// In this workgroup's LDS, for the length of the kernel: set me + x * n_wg is slot x; the node of round r of that
// set (ID = set + r * n_sets) is counter x * rounds + r.
template <typename IdT, int WAYS>
struct StateInLds {
    static constexpr bool in_lds = true;
    IdT* s_tag;
    int32_t* s_stamp;
    uint8_t* s_reuse;
    unsigned long long* s_mm;
    uint32_t rounds, words_per_set;
    FastDiv div_sets;
    LineWordsLds lw;
    char** s_first;                                           // per node of these sets, or nullptr: not kept
    __device__ __forceinline__ char** first_out(uint32_t, uint32_t node) const { return s_first ? s_first + node : nullptr; }
    __device__ __forceinline__ uint32_t slot_of(uint32_t, uint32_t local_set) const { return local_set; }
    __device__ __forceinline__ uint32_t node_of(uint32_t slot, uint32_t round, uint32_t) const { return slot * rounds + round; }
    __device__ __forceinline__ uint32_t node_of_tag(uint32_t slot, uint32_t tag) const {
        return slot * rounds + fast_div(div_sets, tag);
    }
    __device__ __forceinline__ IdT* tags(uint32_t slot) const { return s_tag + slot * WAYS; }
    __device__ __forceinline__ int32_t* stamps(uint32_t slot) const { return s_stamp + slot * WAYS; }
    __device__ __forceinline__ uint8_t* counter(uint32_t node) const { return s_reuse + node; }
    __device__ __forceinline__ unsigned long long* miss_words(uint32_t slot) const { return s_mm + slot * words_per_set; }
    __device__ __forceinline__ uint32_t local_line(uint32_t slot, int way) const { return slot * WAYS + (uint32_t)way; }
};

// List positions out of a stretch of each list that the workgroup took for the whole call (as many places as it
// has entries: none of its entries needs more than one place per list); what is left of a stretch at the end is
// filled with operations that do nothing.
struct PlacesLocal {
    const uint32_t* base;                                     // LDS: the stretches' first places
    uint32_t* used;                                           // LDS: places handed out so far
    __device__ __forceinline__ uint32_t take(int list, uint32_t n) const { return base[list] + atomicAdd(&used[list], n); }
};

// The way a missed ID takes in its set, or -1 when the set has no evictable way left for it: the k-th miss of a
// set (ascending ID) takes the k-th evictable way in (stamp, way) order (seeded hash order under the random
// policy).  Reads the set's stamps, the counters of the nodes it holds and its miss mask as they are now: the
// caller has a barrier between the minibatch's probe and this.
template <typename IdT, int WAYS, typename State>
__device__ __forceinline__ int pick_way(const CacheView<IdT>& c, const State& st, uint32_t slot, uint64_t set,
                                        uint64_t round, int32_t stamp, const IdT (&tg)[WAYS]) {
    const int32_t* sp = st.stamps(slot);
    int32_t stm[WAYS];
#pragma unroll
    for (int w = 0; w < WAYS; w++) stm[w] = sp[w];
    uint8_t ru[WAYS];
#pragma unroll
    for (int w = 0; w < WAYS; w++) ru[w] = tg[w] < 0 ? (uint8_t)0 : *st.counter(st.node_of_tag(slot, (uint32_t)tg[w]));
    uint64_t key[WAYS];
    uint32_t n_ev = 0;
#pragma unroll
    for (int w = 0; w < WAYS; w++) {
        const bool empty = tg[w] < 0;
        const bool ev = stm[w] != stamp && ru[w] == 0;        // untouched in this minibatch, no buffered future use
        uint64_t order = (uint64_t)(uint32_t)(stm[w] + 1);
        if (c.policy == 1)
            order = empty ? 0ull
                          : 1ull + (mix64(mix64(mix64(c.policy_key ^ (uint64_t)(uint32_t)stamp) ^ set) ^ (uint64_t)w) >> 9);
        key[w] = ev ? (order << 8) | (uint64_t)w : ~0ull;
        n_ev += ev;
    }
    uint32_t rank = 0;                                        // of this miss among its set's misses, ascending ID
    const unsigned long long* mm = st.miss_words(slot);
    const uint32_t wi = (uint32_t)(round >> 6);
    for (uint32_t x = 0; x < wi; x++) rank += (uint32_t)__popcll(mm[x]);
    rank += (uint32_t)__popcll(mm[wi] & ((1ull << (round & 63)) - 1));
    if (rank >= n_ev) return -1;
    int way = 0;
#pragma unroll
    for (int w = 0; w < WAYS; w++) {
        uint32_t r = 0;
#pragma unroll
        for (int o = 0; o < WAYS; o++) r += key[o] < key[w];
        if (key[w] != ~0ull && r == rank) way = w;
    }
    return way;
}

// The steps for a workgroup whose share of some list did not fit its LDS: every phase of every step reads the
// whole list from memory again and keeps what it owns; the plan entries pass between the phases through memory.
template <typename IdT, int WAYS>
__device__ void steps_from_memory(const CacheView<IdT>& c, const AccumView& a, uint32_t group, const ManySteps<IdT>& m,
                                  uint64_t* __restrict__ plan_all, uint32_t n_ok, uint32_t stamp0, uint32_t* cnt) {
    Ctl* ctl = c.ctl;
    const uint32_t tid = threadIdx.x;
    const uint32_t n_wg = gridDim.x, me = blockIdx.x;
    if (n_ok && m.pushed[0]) raise_counters(c, m.pushed[0], ctl->win_n[m.pushed_slot[0]], n_wg, me);
    for (uint32_t i = 0; i < n_ok; i++) {
        const int32_t stamp = (int32_t)(stamp0 + i);
        const IdT* __restrict__ U = m.head[i];
        const uint32_t n_u = ctl->win_n[m.head_slot[i]];
        uint64_t* __restrict__ plan = plan_all + m.plan_offset[i];
        if (tid < 5) cnt[tid] = 0;
        // (the list pushed in this step has had its counters raised already: before the loop for step 0,
        // in the previous step's last phase otherwise)
        __syncthreads();
        uint32_t hits = 0, cpus = 0, misses = 0, bypasses = 0, fills = 0;
        // ---- probe: every ID of this workgroup's sets against the state at the start of the minibatch
        for (uint64_t base = tid; base < n_u; base += (uint64_t)blockDim.x * CM_UNROLL) {
            uint64_t vv[CM_UNROLL];
#pragma unroll
            for (int u = 0; u < CM_UNROLL; u++) {
                const uint64_t j = base + (uint64_t)u * blockDim.x;
                vv[u] = j < n_u ? (uint64_t)U[j] : ~0ull;
            }
#pragma unroll
            for (int u = 0; u < CM_UNROLL; u++) {
                const uint64_t j = base + (uint64_t)u * blockDim.x;
                const uint64_t v = vv[u];
                if (v == ~0ull) continue;
                uint64_t set, round;
                set_and_round(c, v, &set, &round);
                if (!owns(c, set, n_wg, me)) continue;
                c.reuse[v] = (uint8_t)(c.reuse[v] - 1);       // this minibatch's own entry leaves the counters
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
                    if ((uint64_t)row[w] == v) way = w;       // empty lines hold -1
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
        __syncthreads();
        // ---- victims
        const bool any_miss = cnt[2] != 0;
        if (any_miss) {
            for (uint64_t base = tid; base < n_u; base += (uint64_t)blockDim.x * CM_UNROLL) {
                uint64_t ee[CM_UNROLL];
#pragma unroll
                for (int u = 0; u < CM_UNROLL; u++) {
                    const uint64_t j = base + (uint64_t)u * blockDim.x;
                    ee[u] = j < n_u ? plan[j] : 0ull;         // (entries of other workgroups' sets are skipped below)
                }
#pragma unroll
                for (int u = 0; u < CM_UNROLL; u++) {
                    const uint64_t j = base + (uint64_t)u * blockDim.x;
                    if (j >= n_u || (ee[u] >> PLAN_SHIFT) != PLAN_MISS_TBD) continue;
                    const uint64_t v = (uint64_t)U[j];
                    uint64_t set, round;
                    set_and_round(c, v, &set, &round);
                    if (!owns(c, set, n_wg, me)) continue;    // (what another workgroup or an earlier call left there)
                    IdT tg[WAYS];
#pragma unroll
                    for (int w = 0; w < WAYS; w++) tg[w] = c.tags[set * WAYS + w];
                    const StateInMemory<IdT, WAYS> st{c, LineWordsGlobal{c.pending, c.fillgrp, c.hitgrp, a.fills[group & 1u]}};
                    const int way = pick_way<IdT, WAYS>(c, st, (uint32_t)set, set, round, stamp, tg);
                    if (way < 0) {
                        plan[j] = PLAN_BYPASS << PLAN_SHIFT;
                        bypasses++;
                    } else {
                        plan[j] = (PLAN_INSTALL << PLAN_SHIFT) | (set * WAYS + (uint32_t)way);
                        fills++;
                    }
                }
            }
            __syncthreads();
        }
        // ---- publish tags and stamps, clear the miss mask, queue every row into the open group's lists
        for (uint64_t base = 0; base < n_u; base += blockDim.x) {     // uniform trip count: queue_entry ballots
            const uint64_t j = base + tid;
            bool mine = false;
            uint64_t e = 0, v = 0;
            if (j < n_u) {
                v = (uint64_t)U[j];
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
            queue_entry(c, a, group, mine, j, e, v, m.out[i], m.unique_out[i]);
        }
        // the next step's pushed list enters the counters now: this step's victims are chosen, and the next
        // step's probe, which must see them, waits behind a barrier
        if (i + 1 < m.k && m.pushed[i + 1]) raise_counters(c, m.pushed[i + 1], ctl->win_n[m.pushed_slot[i + 1]], n_wg, me);
        // ---- this workgroup's share of the step's counters
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
        if (tid < 5 && cnt[tid]) atomicAdd(&ctl->many_cnt[i][tid], cnt[tid]);
        __syncthreads();                                      // cnt is cleared at the top of the next step
    }
}

// The barrier between two phases of a step.  With the state in LDS a phase reads nothing from device memory that
// the kernel writes, so only the LDS traffic has to be through: the stores to the group's lists and to the
// callers' buffers stay in flight (beside a row mover that saturates the host link their acknowledgements take
// microseconds).
template <bool LDS_ONLY>
__device__ __forceinline__ void phase_barrier() {
    if constexpr (LDS_ONLY) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    } else {
        __syncthreads();
    }
}

// CPU-buffer lookup (Section 3.3): the row of the buffer that holds node v, or CM_NONE
template <typename IdT>
__device__ __forceinline__ uint32_t cpu_row_of(const CacheView<IdT>& c, uint64_t v) {
    if (!c.hotbits) return CM_NONE;
    const uint64_t hw = c.hotbits[v >> 6];
    const uint32_t before = c.hotrank[v >> 6];                // (both loads at once)
    const uint64_t bit = 1ull << (v & 63);
    return (hw & bit) ? before + (uint32_t)__popcll(hw & (bit - 1)) : CM_NONE;
}

// one wavefront's count of a flag, added to a counter in LDS
__device__ __forceinline__ void wave_count(uint32_t* counter, bool flag) {
    const uint64_t b = __ballot(flag);
    if (b && (threadIdx.x & 63) == 0) atomicAdd(counter, (uint32_t)__popcll(b));
}

// The steps for a workgroup whose entries of every list are in its LDS pool: one thread per entry, and what it
// learns of its entry stays in its registers from phase to phase.  Between the phases only workgroup barriers:
// what a phase reads was written by this same workgroup (its sets' tags, stamps and miss masks, its nodes'
// counters, its own list operations), and a barrier orders memory within a workgroup.
template <typename IdT, int WAYS, typename State>
__device__ __forceinline__ void steps_from_pool(const CacheView<IdT>& c, const AccumView& a, const State& st,
                                                uint32_t group, const ManySteps<IdT>& m, uint32_t n_ok, uint32_t stamp0,
                                                const uint32_t* pool_v, const uint32_t* pool_j, const uint32_t* pool_cpu,
                                                const uint32_t* own_n, uint32_t (*cnt)[6], const PlacesLocal& places) {
    const uint32_t tid = threadIdx.x;
    const uint32_t cap = m.share_cap;
    const uint32_t n_sets = (uint32_t)c.n_sets;
    // the list pushed in step 0: one more buffered future use for each of its nodes (Section 3.4, Fig. 6)
    if (m.pushed_list[0] != MANY_NO_LIST && tid < own_n[m.pushed_list[0]]) {
        const uint32_t pv = pool_v[(size_t)m.pushed_list[0] * cap + tid];
        const uint32_t round = fast_div(m.div_sets, pv), set = pv - round * n_sets;
        uint8_t* ctr = st.counter(st.node_of(st.slot_of(set, set >> m.wg_shift), round, pv));
        *ctr = (uint8_t)(*ctr + 1);
    }
    phase_barrier<State::in_lds>();
    for (uint32_t i = 0; i < n_ok; i++) {
        const int32_t stamp = (int32_t)(stamp0 + i);
        const uint32_t h = m.head_list[i];
        const uint32_t n_h = own_n[h];
        const bool have = tid < n_h;
        const bool wave_has = (tid & ~63u) < n_h;
        uint64_t e = 0;
        uint32_t v = 0, j = 0, set = 0, round = 0, slot = 0, local = 0;
        char** first = nullptr;
        bool miss = false;
        IdT tg[WAYS];
#pragma unroll
        for (int w = 0; w < WAYS; w++) tg[w] = (IdT)-1;
        // ---- probe, against the state at the start of the minibatch
        if (have) {
            v = pool_v[(size_t)h * cap + tid];
            j = pool_j[(size_t)h * cap + tid];
            // (looked up once per call where the pool has room for it, here otherwise)
            const uint32_t cpu_row = pool_cpu ? pool_cpu[(size_t)h * cap + tid] : cpu_row_of(c, v);
            round = fast_div(m.div_sets, v);
            set = v - round * n_sets;
            slot = st.slot_of(set, set >> m.wg_shift);
            const uint32_t node = st.node_of(slot, round, v);
            uint8_t* ctr = st.counter(node);
            const uint8_t r = *ctr;
            if (cpu_row != CM_NONE) {
                e = (PLAN_CPU << PLAN_SHIFT) | cpu_row;
                if (m.group_dedup) first = st.first_out(cpu_row, node);
            } else {
                const IdT* row = st.tags(slot);
                int way = -1;
#pragma unroll
                for (int w = 0; w < WAYS; w++) {
                    tg[w] = row[w];
                    if ((uint64_t)tg[w] == (uint64_t)v) way = w;   // empty lines hold -1
                }
                if (way >= 0) {
                    st.stamps(slot)[way] = stamp;
                    e = (PLAN_HIT << PLAN_SHIFT) | ((uint64_t)set * WAYS + (uint32_t)way);
                    local = st.local_line(slot, way);
                } else {
                    miss = true;
                    e = PLAN_MISS_TBD << PLAN_SHIFT;
                    atomicOr(st.miss_words(slot) + (round >> 6), 1ull << (round & 63));
                }
            }
            *ctr = (uint8_t)(r - 1);                          // this minibatch's own entry leaves the counters
        }
        if (wave_has) {
            wave_count(&cnt[i][0], have && (e >> PLAN_SHIFT) == PLAN_HIT);
            wave_count(&cnt[i][1], have && (e >> PLAN_SHIFT) == PLAN_CPU);
            wave_count(&cnt[i][2], miss);
        }
        phase_barrier<State::in_lds>();
        // ---- victims
        if (cnt[i][2]) {
            if (miss) {
                const int way = pick_way<IdT, WAYS>(c, st, slot, (uint64_t)set, (uint64_t)round, stamp, tg);
                if (way < 0) {
                    e = PLAN_BYPASS << PLAN_SHIFT;
                } else {
                    e = (PLAN_INSTALL << PLAN_SHIFT) | ((uint64_t)set * WAYS + (uint32_t)way);
                    local = st.local_line(slot, way);
                }
            }
            if (wave_has) {
                wave_count(&cnt[i][3], miss && (e >> PLAN_SHIFT) == PLAN_BYPASS);
                wave_count(&cnt[i][4], miss && (e >> PLAN_SHIFT) == PLAN_INSTALL);
            }
            phase_barrier<State::in_lds>();
        }
        // ---- publish tags and stamps, clear the miss mask, queue every row into the open group's lists; the
        // next step's pushed list enters the counters: this step's victims are chosen, and the next step's
        // probe, which must see them, waits behind the barrier
        const uint32_t pl = i + 1 < m.k ? m.pushed_list[i + 1] : MANY_NO_LIST;
        if (pl != MANY_NO_LIST && tid < own_n[pl]) {
            const uint32_t pv = pool_v[(size_t)pl * cap + tid];
            const uint32_t pr = fast_div(m.div_sets, pv), ps = pv - pr * n_sets;
            uint8_t* ctr = st.counter(st.node_of(st.slot_of(ps, ps >> m.wg_shift), pr, pv));
            *ctr = (uint8_t)(*ctr + 1);
        }
        if (miss) {
            if ((e >> PLAN_SHIFT) == PLAN_INSTALL) {
                const uint32_t way = (uint32_t)(e & PLAN_INDEX_MASK) - set * WAYS;
                st.tags(slot)[way] = (IdT)v;
                st.stamps(slot)[way] = stamp;
            }
            st.miss_words(slot)[round >> 6] = 0ull;
        }
        if (wave_has) {
            const bool again = queue_entry(c, a, st.lw, places, group, have, (uint64_t)j, e, (uint64_t)v, local, m.out[i],
                                           m.unique_out[i], first);
            if (m.group_dedup) wave_count(&cnt[i][5], again);
        }
        phase_barrier<State::in_lds>();
    }
}

template <typename IdT, int WAYS>
__global__ __launch_bounds__(CM_THREADS) void classify_many_kernel(CacheView<IdT> c, AccumView a, uint32_t group,
                                                                   ManySteps<IdT> m, uint64_t* __restrict__ plan_all,
                                                                   StatsRec* ring, uint32_t ring_size) {
    // Dynamic LDS.  The pool: this workgroup's entries of every list of the launch, picked out once: share_cap places
    // per list (ID, position in the list), filled in no particular order.  With m.resident, also the entries'
    // CPU-buffer rows (or CM_NONE), the state of this workgroup's sets and nodes for the length of the kernel and,
    // with m.group_dedup, a word per node for the output row of the call's first fill of it.
    extern __shared__ unsigned long long lds_raw[];
    __shared__ uint32_t list_n[2 * MANY_MAX];                 // entries of each list
    __shared__ uint32_t list_off[2 * MANY_MAX + 1];           // entries of the lists before it
    __shared__ const IdT* list_ptr[2 * MANY_MAX];
    __shared__ uint32_t own_n[2 * MANY_MAX];                  // of which this workgroup's
    __shared__ uint32_t cnt[MANY_MAX][6];                     // per step: hits, CPU-buffer hits, misses, bypasses, line fills, CPU rows by copy
    __shared__ uint32_t cnt_mem[5];
    __shared__ uint32_t overflow;
    __shared__ uint32_t is_last;
    __shared__ uint32_t place_base[3], place_used[3], place_n;
    Ctl* ctl = c.ctl;
    // A chain of short dependent steps: where it shares a compute unit with wavefronts of a row mover, it goes first.
    __builtin_amdgcn_s_setprio(3);
    const uint32_t tid = threadIdx.x;
    const uint32_t n_wg = gridDim.x, me = blockIdx.x;
    const uint32_t stamp0 = ctl->stamp;
    const uint32_t cap = m.share_cap;
    const uint32_t n_sets = (uint32_t)c.n_sets;
    const uint32_t spw = m.resident ? m.sets_per_wg : 0;      // places for sets, their lines, miss-mask words, nodes
    const uint32_t n_l = spw * WAYS, n_mw = spw * c.words_per_set, n_nodes = spw * m.rounds;
    const size_t n_pool = (size_t)m.n_lists * cap;
    const uint32_t n_first = m.group_dedup ? n_nodes : 0;     // (only with the state in LDS: spw is 0 otherwise)
    char** s_pout = reinterpret_cast<char**>(lds_raw);
    char** s_first = s_pout + n_l;
    unsigned long long* s_mm = lds_raw + n_l + n_first;
    IdT* s_tag = reinterpret_cast<IdT*>(s_mm + n_mw);
    uint32_t* pool_v = reinterpret_cast<uint32_t*>(s_tag + n_l);
    uint32_t* pool_j = pool_v + n_pool;
    // (the CPU-buffer row of an entry is kept only beside the sets' state: where that stays in memory the steps
    // wait for memory anyway, and the room goes to longer lists or more steps per call)
    uint32_t* pool_cpu = m.resident ? pool_j + n_pool : nullptr;
    int32_t* s_stamp = reinterpret_cast<int32_t*>(pool_j + n_pool + (m.resident ? n_pool : 0));
    uint32_t* s_pend = reinterpret_cast<uint32_t*>(s_stamp + n_l);
    uint32_t* s_fgrp = s_pend + n_l;
    uint32_t* s_hgrp = s_fgrp + n_l;
    uint8_t* s_reuse = reinterpret_cast<uint8_t*>(s_hgrp + n_l);

    for (uint32_t l = tid; l < m.n_lists; l += blockDim.x) {
        list_n[l] = ctl->win_n[m.list_slot[l]];
        list_ptr[l] = m.list[l];
        own_n[l] = 0;
    }
    for (uint32_t x = tid; x < MANY_MAX * 6; x += blockDim.x) cnt[x / 6][x % 6] = 0;
    if (tid == 0) overflow = cap == 0;
    __syncthreads();
    // an error left by an earlier kernel (a pushed ID out of range): nothing runs, every record reports it.
    // A step whose list exceeds its output: the same verdict in every workgroup, it and the later ones do not run.
    uint32_t n_ok = ld_agent(&ctl->error) == 0 ? m.k : 0;
    for (uint32_t i = 0; i < n_ok; i++)
        if (list_n[m.head_list[i]] > m.out_capacity[i]) n_ok = i;
    if (tid == 0) {
        uint32_t off = 0;
        for (uint32_t l = 0; l < m.n_lists; l++) {
            list_off[l] = off;
            off += list_n[l];
        }
        list_off[m.n_lists] = off;
    }
    __syncthreads();

    // ---- every list once: the IDs of this workgroup's sets go to its LDS.  The lists are read as one long
    // sequence, eight entries per thread in flight whichever lists they fall into: the pass waits for memory a
    // few times, not once per list.
    if (cap && n_ok) {
        const uint32_t total = list_off[m.n_lists];
        uint32_t l = 0;                                       // the list this thread's next entry falls into
        for (uint32_t f0 = tid; f0 < total; f0 += blockDim.x * CM_SCAN) {
            uint32_t vv[CM_SCAN], jj[CM_SCAN], ll[CM_SCAN];
#pragma unroll
            for (int u = 0; u < CM_SCAN; u++) {
                const uint32_t f = f0 + (uint32_t)u * blockDim.x;
                vv[u] = ~0u;
                if (f < total) {
                    while (f >= list_off[l + 1]) l++;
                    ll[u] = l;
                    jj[u] = f - list_off[l];
                    vv[u] = (uint32_t)list_ptr[l][jj[u]];     // (a table of this kind has far fewer than 2^32 rows)
                }
            }
#pragma unroll
            for (int u = 0; u < CM_SCAN; u++) {
                if (vv[u] == ~0u) continue;
                const uint32_t set = vv[u] - fast_div(m.div_sets, vv[u]) * n_sets;
                if ((set & (n_wg - 1)) != me) continue;       // (the number of workgroups is a power of two)
                const uint32_t pos = atomicAdd(&own_n[ll[u]], 1u);
                if (pos < cap) {
                    pool_v[(size_t)ll[u] * cap + pos] = vv[u];
                    pool_j[(size_t)ll[u] * cap + pos] = jj[u];
                } else {
                    overflow = 1;
                }
            }
        }
    }
    __syncthreads();
    const bool from_memory = overflow != 0;                   // the same in every thread of the workgroup
    if (from_memory) {
        steps_from_memory<IdT, WAYS>(c, a, group, m, plan_all, n_ok, stamp0, cnt_mem);
    } else if (n_ok) {
        // A stretch of each of the group's lists for this workgroup's entries, taken once: three atomics per
        // workgroup and call instead of three per wavefront and step.
        if (tid == 0) {
            uint32_t n = 0;
            for (uint32_t i = 0; i < n_ok; i++) n += own_n[m.head_list[i]];
            const uint32_t par = group & 1u;
            place_n = n;
            place_base[0] = atomicAdd(&ctl->q_fill[par], n);
            place_base[1] = atomicAdd(&ctl->q_rcopy[par], n);
            place_base[2] = atomicAdd(&ctl->q_wcopy[par], n);
            place_used[0] = place_used[1] = place_used[2] = 0;
        }
        const PlacesLocal places{place_base, place_used};
        // CPU-buffer lookup (Section 3.3) of every entry that will be gathered: the buffer is constant
        // (list_off is free again: now the workgroup's entries of the lists before a list, gathered lists only)
        if (tid == 0) {
            uint32_t off = 0;
            for (uint32_t l = 0; l < m.n_lists; l++) {
                list_off[l] = off;
                off += m.list_is_head[l] ? own_n[l] : 0u;
            }
            list_off[m.n_lists] = off;
        }
        __syncthreads();
        if (pool_cpu) {
            const uint32_t total = list_off[m.n_lists];
            uint32_t l = 0;
            for (uint32_t f = tid; f < total; f += blockDim.x) {
                while (f >= list_off[l + 1]) l++;
                const uint32_t x = l * cap + (f - list_off[l]);
                pool_cpu[x] = cpu_row_of(c, (uint64_t)pool_v[x]);
            }
        }
        if (m.resident) {
            // ---- the state of this workgroup's sets and nodes comes into LDS (the miss masks are clear
            // between gathers)
            for (uint32_t x = tid; x < n_l; x += blockDim.x) {
                const uint32_t set = me + (x / WAYS) * n_wg;
                if (set >= n_sets) continue;
                const uint64_t line = (uint64_t)set * WAYS + x % WAYS;
                s_tag[x] = c.tags[line];
                s_stamp[x] = c.stamps[line];
                s_pend[x] = c.pending[line];
                s_fgrp[x] = c.fillgrp[line];
                s_hgrp[x] = c.hitgrp[line];
                s_pout[x] = nullptr;                          // (read only for fills queued by this call's group)
            }
            for (uint32_t x = tid; x < n_mw; x += blockDim.x) s_mm[x] = 0ull;
            for (uint32_t x = tid; x < n_first; x += blockDim.x) s_first[x] = nullptr;
            for (uint32_t x = tid; x < n_nodes; x += blockDim.x) {
                const uint32_t ls = x / m.rounds;
                const uint64_t v = (uint64_t)(me + ls * n_wg) + (uint64_t)(x - ls * m.rounds) * n_sets;
                if (me + ls * n_wg < n_sets && v < c.n_rows) s_reuse[x] = c.reuse[v];
            }
            __syncthreads();
            const StateInLds<IdT, WAYS> st{s_tag, s_stamp, s_reuse, s_mm, m.rounds, c.words_per_set, m.div_sets,
                                           LineWordsLds{s_pend, s_fgrp, s_hgrp, s_pout}, n_first ? s_first : nullptr};
            steps_from_pool<IdT, WAYS>(c, a, st, group, m, n_ok, stamp0, pool_v, pool_j, pool_cpu, own_n, cnt, places);
            // ---- the fills that still wait in the lines' words are queued (steps_from_pool ends behind a barrier)
            for (uint32_t x = tid; x < n_l; x += blockDim.x) {
                const uint32_t set = me + (x / WAYS) * n_wg;
                if (set >= n_sets || s_fgrp[x] != group) continue;
                const uint64_t line = (uint64_t)set * WAYS + x % WAYS;
                const uint32_t node = s_pend[x] & 0x7FFFFFFFu;
                const bool late = (s_pend[x] >> 31) != 0;
                const uint32_t par = group & 1u;
                const uint32_t q = places.take(0, 1u);
                if (q < a.cap) {
                    FillOp op;
                    op.src = c.store + (uint64_t)node * c.row_bytes;
                    op.dst_out = s_pout[x];
                    op.dst_line = late ? NO_LINE : line;
                    op.late = NO_OP;
                    op.pad = 0;
                    a.fills[par][q] = op;
                }
                if (late) {                                   // after the rcopies that still read the line's old bytes
                    const uint32_t w = places.take(2, 1u);
                    if (w < a.cap) a.wcopies[par][w] = CopyOp{s_pout[x], c.cache_data + line * c.line_bytes};
                }
                s_pend[x] = q;                                // what the per-step kernels leave there: the fill's place
            }
            __syncthreads();
            // ---- and the state goes back
            for (uint32_t x = tid; x < n_l; x += blockDim.x) {
                const uint32_t set = me + (x / WAYS) * n_wg;
                if (set >= n_sets) continue;
                const uint64_t line = (uint64_t)set * WAYS + x % WAYS;
                c.tags[line] = s_tag[x];
                c.stamps[line] = s_stamp[x];
                c.pending[line] = s_pend[x];
                c.fillgrp[line] = s_fgrp[x];
                c.hitgrp[line] = s_hgrp[x];
            }
            for (uint32_t x = tid; x < n_nodes; x += blockDim.x) {
                const uint32_t ls = x / m.rounds;
                const uint64_t v = (uint64_t)(me + ls * n_wg) + (uint64_t)(x - ls * m.rounds) * n_sets;
                if (me + ls * n_wg < n_sets && v < c.n_rows) c.reuse[v] = s_reuse[x];
            }
        } else {
            __syncthreads();
            const StateInMemory<IdT, WAYS> st{c, LineWordsGlobal{c.pending, c.fillgrp, c.hitgrp, a.fills[group & 1u]}};
            steps_from_pool<IdT, WAYS>(c, a, st, group, m, n_ok, stamp0, pool_v, pool_j, pool_cpu, own_n, cnt, places);
            if (m.group_dedup && c.cpu_first && m.step0 == 0 && m.closes_group) {
                // the words that remember the call's first fill of a CPU-buffer row are clear between calls
                // (a call in several launches: the host clears the table behind the last)
                // (list_off still holds this workgroup's entries of the gathered lists)
                const uint32_t total = list_off[m.n_lists];
                uint32_t l = 0;
                for (uint32_t f = tid; f < total; f += blockDim.x) {
                    while (f >= list_off[l + 1]) l++;
                    const uint32_t row = cpu_row_of(c, (uint64_t)pool_v[l * cap + (f - list_off[l])]);
                    if (row != CM_NONE) c.cpu_first[row] = nullptr;
                }
            }
        }
        for (uint32_t x = tid; x < m.k * 6; x += blockDim.x)
            if (cnt[x / 6][x % 6]) atomicAdd(&ctl->many_cnt[x / 6][x % 6], cnt[x / 6][x % 6]);
        // what is left of the three stretches: operations that do nothing (the host sizes each list for every
        // entry of the group, so the stretches always fit; were one to end beyond its list, queue_entry has
        // reported it and nothing is written there)
        {
            const uint32_t par = group & 1u;
            const uint64_t end = a.cap;
            FillOp none;
            none.src = nullptr; none.dst_out = nullptr; none.dst_line = NO_LINE; none.late = NO_OP; none.pad = 0;
            for (uint64_t x = (uint64_t)place_base[0] + place_used[0] + tid; x < (uint64_t)place_base[0] + place_n && x < end; x += blockDim.x)
                a.fills[par][x] = none;
            for (uint64_t x = (uint64_t)place_base[1] + place_used[1] + tid; x < (uint64_t)place_base[1] + place_n && x < end; x += blockDim.x)
                a.rcopies[par][x] = CopyOp{nullptr, nullptr};
            for (uint64_t x = (uint64_t)place_base[2] + place_used[2] + tid; x < (uint64_t)place_base[2] + place_n && x < end; x += blockDim.x)
                a.wcopies[par][x] = CopyOp{nullptr, nullptr};
        }
        __syncthreads();
    }
    // ---- the last workgroup to get here publishes the records
    if (tid == 0) {
        __threadfence();
        is_last = atomicAdd(&ctl->ticket_cls, 1u) == n_wg - 1;
    }
    __syncthreads();
    if (!is_last) return;
    // (one thread per record: the counters of a step are five loads that wait for nothing but each other)
    if (tid == 0) {
        __threadfence();
        if (n_ok < m.k && ld_agent(&ctl->error) == 0) atomicCAS(&ctl->error, 0u, 7u /* -GIDS_E_SPACE: step n_ok's output */);
    }
    __syncthreads();
    const uint32_t err = ld_agent(&ctl->error);
    if (tid < m.k) {
        const uint32_t i = tid;
        StatsRec* rec = ring + (m.seq0 + i) % ring_size;
        const bool ran = i < n_ok;
        const uint32_t n = ran ? list_n[m.head_list[i]] : 0u;
        uint32_t queued = (m.step0 ? ctl->q_rows : 0u) + n;     // (rows the call's earlier launches queued)
        for (uint32_t x = 0; x < i && x < n_ok; x++) queued += list_n[m.head_list[x]];
        rec->n_unique = n;
        rec->n_hit = ld_agent(&ctl->many_cnt[i][0]);
        rec->n_cpu_hit = ld_agent(&ctl->many_cnt[i][1]);
        rec->n_miss = ld_agent(&ctl->many_cnt[i][2]);
        rec->n_bypass = ld_agent(&ctl->many_cnt[i][3]);
        rec->n_line_fills = ld_agent(&ctl->many_cnt[i][4]);
        rec->n_cpu_again = ld_agent(&ctl->many_cnt[i][5]);
        const bool closes = m.closes_group && i + 1 == m.k;   // the call's steps are one group, closed by its last
        rec->n_pending = closes ? 0u : queued;
        rec->flushed = closes ? 1 : 0;
        rec->status = ran ? 0 : -(int32_t)err;
        ctl->grp_nu[group & 1u][m.step0 + i] = n;
        for (int x = 0; x < 6; x++) ctl->many_cnt[i][x] = 0;
    }
    __syncthreads();                                          // (every record has read the rows queued before)
    if (tid == 0) {
        uint32_t all = m.step0 ? ctl->q_rows : 0u;
        for (uint32_t x = 0; x < n_ok; x++) all += list_n[m.head_list[x]];
        ctl->q_rows = m.closes_group ? 0u : all;
        ctl->stamp = stamp0 + n_ok;
        ctl->ticket_cls = 0;
    }
    __threadfence_system();
    __syncthreads();
    if (tid < m.k) ring[(m.seq0 + tid) % ring_size].seq = m.seq0 + tid;   // a record whose seq matches is complete
    __threadfence_system();
}

}  // namespace

// rows whose bitmap fits the LDS one workgroup may take on the current device (all of a CU's on gfx950)
uint64_t many_max_rows() {
    static const uint64_t rows = [] {
        int dev = 0, lds = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess || lds < 65536) {
            (void)hipGetLastError();
            lds = 65536;
        }
        return (uint64_t)(lds - 1024) * 8;                   // 1 KiB left for the kernel's other shared variables
    }();
    return rows;
}
uint32_t many_max_ways() { return 16; }

template <typename IdT>
void launch_dedup_small(const ManyPushes<IdT>& p, uint32_t n_lists, uint64_t n_rows, Ctl* ctl, hipStream_t s) {
    if (n_lists == 0) return;
    const size_t lds = (size_t)((n_rows + 63) / 64) * sizeof(unsigned long long);
    static bool raised = false;                               // more than the default 64 KiB has to be asked for, once
    if (lds > 65536 && !raised) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&dedup_small_kernel<IdT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)(many_max_rows() / 8));
        raised = true;
    }
    hipLaunchKernelGGL(dedup_small_kernel<IdT>, dim3(n_lists), dim3(DS_THREADS), lds, s, p, n_rows, ctl);
}

namespace {
template <typename IdT, int W>
void launch_classify_many_ways(const CacheView<IdT>& c, const AccumView& a, uint32_t group, const ManySteps<IdT>& m,
                               uint32_t grid, uint32_t threads, size_t lds, uint64_t* plan_all, StatsRec* ring,
                               uint32_t ring_size, hipStream_t s) {
    static bool raised = false;                               // more than the default 64 KiB has to be asked for, once
    if (lds > 49152 && !raised) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&classify_many_kernel<IdT, W>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)MANY_LDS_MAX_BYTES);
        raised = true;
    }
    hipLaunchKernelGGL((classify_many_kernel<IdT, W>), dim3(grid), dim3(threads), lds, s, c, a, group, m, plan_all,
                       ring, ring_size);
}
}  // namespace

namespace {
// How a merged call's classification is launched: workgroups, their threads, and what their LDS holds.
struct ManyShape {
    uint64_t g;             // workgroups, a power of two
    uint32_t wg_shift;
    uint32_t threads;
    uint32_t sets_per_wg, rounds;
    uint64_t state;         // bytes of a workgroup's sets' state
    bool resident;          // ... kept in LDS for the length of the kernel
    uint64_t cap;           // places per list for a workgroup's own entries
    uint64_t share;         // entries of the longest list a workgroup can expect to own
};

ManyShape many_shape(uint64_t n_rows, uint64_t n_sets, uint32_t ways, uint32_t words_per_set, size_t id_bytes,
                     uint32_t n_lists, uint64_t longest, uint64_t pool_bytes, bool group_dedup) {
    // 16 to 32 of a list's entries per workgroup's own share (GIDS_MANY_SHARE); every workgroup reads every list
    static const uint64_t per_wg = [] {
        const char* e = getenv("GIDS_MANY_SHARE");
        const long v = e ? atol(e) : 16;
        return (uint64_t)(v >= 1 ? v : 16);
    }();
    static const uint32_t threads = [] {                     // a multiple of 64 up to CM_THREADS (GIDS_MANY_THREADS)
        const char* e = getenv("GIDS_MANY_THREADS");
        const long v = e ? atol(e) : CM_THREADS;
        return (uint32_t)(v >= 64 && v <= CM_THREADS ? v & ~63l : CM_THREADS);
    }();
    static const bool resident_ok = [] {                      // GIDS_MANY_RESIDENT=0: the sets' state stays in memory
        const char* e = getenv("GIDS_MANY_RESIDENT");
        return !(e && atoi(e) == 0);
    }();
    ManyShape sh;
    uint64_t g = (longest + per_wg - 1) / per_wg;
    if (g < 1) g = 1;
    if (g > 256) g = 256;
    if (g > n_sets) g = n_sets;                               // a workgroup without a set would only take a ticket
    sh.wg_shift = 0;                                          // a power of two: which workgroup a set belongs to and
    while ((2ull << sh.wg_shift) <= g) sh.wg_shift++;         // its place there are a mask and a shift
    sh.g = 1ull << sh.wg_shift;
    sh.threads = threads;
    // The state of a workgroup's sets for the length of the kernel, when it leaves at least half of the LDS to
    // the lists: per line a tag, a stamp, three accumulator words and an output address; per set its miss-mask
    // words; per node that maps to one of the sets a counter.
    sh.sets_per_wg = (uint32_t)((n_sets + sh.g - 1) / sh.g);
    sh.rounds = (uint32_t)((n_rows + n_sets - 1) / n_sets);
    const uint64_t n_l = (uint64_t)sh.sets_per_wg * ways;
    sh.state = n_l * (8 + id_bytes + 16) + (uint64_t)sh.sets_per_wg * words_per_set * 8 +
               (uint64_t)sh.sets_per_wg * sh.rounds * (group_dedup ? 9 : 1);   // (+ an output address per node)
    sh.resident = resident_ok && pool_bytes && sh.state <= MANY_LDS_MAX_BYTES / 2;
    // LDS for a workgroup's own entries: the same number of places for each list, four times the expected share
    // where that fits; a workgroup whose share of some list is larger reads the lists from memory instead
    const uint64_t room = MANY_LDS_MAX_BYTES - (sh.resident ? sh.state : 0) - 16;
    if (pool_bytes > room) pool_bytes = room;
    const uint64_t entry = sh.resident ? 12 : 8;              // ID (as 32 bits), position in its list; CPU-buffer row
    sh.share = (longest + sh.g - 1) / sh.g;
    uint64_t cap = n_lists ? pool_bytes / (entry * n_lists) : 0;
    if (cap > 4 * sh.share + 16) cap = 4 * sh.share + 16;
    if (cap > threads) cap = threads;                         // one thread per entry
    sh.cap = cap & ~1ull;                                     // keeps the 32-bit arrays behind the IDs aligned
    return sh;
}
}  // namespace

// Whether the merged kernels suit a call: the workgroups' LDS has room for their expected share of every list and
// four standard deviations more (a share is a count of independent hits on one of g residues).  Beyond that most
// workgroups would read the lists from memory in every phase, and the per-step kernels are the better choice.
bool many_fits(uint64_t n_rows, uint64_t n_sets, uint32_t ways, uint32_t words_per_set, size_t id_bytes, uint32_t n_lists,
               uint64_t longest, uint64_t pool_bytes, bool group_dedup, bool* state_in_lds) {
    const ManyShape sh = many_shape(n_rows, n_sets, ways, words_per_set, id_bytes, n_lists, longest, pool_bytes, group_dedup);
    if (state_in_lds) *state_in_lds = sh.resident;
    uint64_t dev = 0;
    while ((dev + 1) * (dev + 1) <= sh.share) dev++;          // floor(sqrt(share))
    return pool_bytes == 0 || sh.cap >= sh.share + 4 * (dev + 1) + 8;
}

template <typename IdT>
void launch_classify_many(const CacheView<IdT>& c, const AccumView& a, uint32_t group, ManySteps<IdT>& m,
                          uint64_t longest, uint64_t pool_bytes, uint64_t* plan_all, StatsRec* ring, uint32_t ring_size,
                          hipStream_t s) {
    const ManyShape sh = many_shape(c.n_rows, c.n_sets, c.ways, c.words_per_set, sizeof(IdT), m.n_lists, longest, pool_bytes,
                                    m.group_dedup != 0);
    const uint64_t g = sh.g;
    const uint32_t threads = sh.threads;
    m.wg_shift = sh.wg_shift;
    m.div_sets = make_fast_div((uint32_t)c.n_sets);
    m.sets_per_wg = sh.sets_per_wg;
    m.rounds = sh.rounds;
    m.resident = sh.resident;
    m.share_cap = (uint32_t)sh.cap;
    const size_t lds = (size_t)(sh.cap * m.n_lists * (sh.resident ? 12 : 8) + (sh.resident ? sh.state : 0) + 16);
#define GIDS_CLASSIFY_MANY(W) \
    launch_classify_many_ways<IdT, W>(c, a, group, m, (uint32_t)g, threads, lds, plan_all, ring, ring_size, s)
    switch (c.ways) {
        case 1: GIDS_CLASSIFY_MANY(1); break;
        case 2: GIDS_CLASSIFY_MANY(2); break;
        case 4: GIDS_CLASSIFY_MANY(4); break;
        case 8: GIDS_CLASSIFY_MANY(8); break;
        default: GIDS_CLASSIFY_MANY(16); break;
    }
#undef GIDS_CLASSIFY_MANY
}

#define GIDS_INSTANTIATE(IdT)                                                                                     \
    template void launch_dedup_small<IdT>(const ManyPushes<IdT>&, uint32_t, uint64_t, Ctl*, hipStream_t);         \
    template void launch_classify_many<IdT>(const CacheView<IdT>&, const AccumView&, uint32_t, ManySteps<IdT>&,  \
                                            uint64_t, uint64_t, uint64_t*, StatsRec*, uint32_t, hipStream_t);
GIDS_INSTANTIATE(int32_t)
GIDS_INSTANTIATE(int64_t)

}  // namespace gids
