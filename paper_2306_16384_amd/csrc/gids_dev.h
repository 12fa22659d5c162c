// Internal declarations shared by the library's translation units: the
// device-resident control block, the plan encoding, and the host-side launchers
// of every kernel.  Nothing here is part of the C ABI (see include/gids.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gids {

// ---- plan entry: what the row mover does for the j-th distinct ID ----------
// bits 63..61 = kind, bits 60..0 = cache line index (HIT, INSTALL) or CPU-buffer
// slot (CPU); BYPASS, FOLLOW and MISS_TBD carry no index.  FOLLOW exists only with several rows per cache
// line: a miss whose line another ID of the same minibatch fills; its own row comes from the store.
constexpr uint64_t PLAN_HIT = 0, PLAN_CPU = 1, PLAN_INSTALL = 2, PLAN_BYPASS = 3, PLAN_MISS_TBD = 4, PLAN_FOLLOW = 5;
constexpr int PLAN_SHIFT = 61;
constexpr uint64_t PLAN_INDEX_MASK = (1ull << PLAN_SHIFT) - 1;

constexpr uint32_t NO_OP = 0xFFFFFFFFu;       // "no pending fill" marker of a cache line
constexpr uint64_t NO_LINE = ~0ull;           // a queued fill that installs nothing

constexpr int MANY_MAX = 32;                // steps one merged call can bring
constexpr int MAX_WINDOW_SLOTS = 256 + MANY_MAX;   // window_depth <= 254, + 2, + the lists a merged call pushes at once

// Device-resident control block of one cache.  Kernels read every count from
// here, so the host never has to wait for a count before launching the next.
struct Ctl {
    uint32_t n_unique;      // distinct IDs of the list deduplicated last
    uint32_t error;         // first error a kernel found (-GIDS_E_*), 0 = none; sticky
    uint32_t ticket;        // arrival counter for "last block does the scan"
    uint32_t ticket_flush;  // ... for "last block of the group mover empties the group's lists"
    uint32_t ticket_cls;    // ... for "last block of the settle kernel publishes the counters"
    uint32_t stamp;         // index of the minibatch being gathered (successful gathers so far)
    uint32_t cnt_hit, cnt_cpu, cnt_miss, cnt_bypass;
    uint32_t cnt_fill;      // cache lines this minibatch fills
    uint32_t cnt_again;     // CPU-buffer rows this minibatch receives as copies of an earlier fill of its group
    // accumulator: rows of the minibatches merged so far (the open group), and the lengths of the three
    // operation lists of the two groups that can exist at a time (the open one and the one being moved)
    uint32_t q_rows;
    uint32_t q_fill[2];     // rows that cross the host link
    uint32_t q_rcopy[2];    // hits whose line already holds its bytes
    uint32_t q_wcopy[2];    // copies that must follow the link rows: hits on lines filled in the same group, ...
    uint32_t q_chunk[2];    // work counter of the group mover's link half
    uint32_t grp_nu[2][MANY_MAX];   // distinct count of each minibatch of a group, in the group's order
    uint32_t many_cnt[MANY_MAX][6];     // per step of a merged call: hits, CPU-buffer hits, misses, bypasses, line fills, CPU-buffer rows by copy
    uint32_t win_n[MAX_WINDOW_SLOTS];   // distinct count of each buffered list
};

// What the row mover needs to know about one gather, frozen by the commit
// kernel so that the next gather's metadata kernels may already run while the
// rows of this one are still moving.
struct BatchHdr {
    uint32_t ok;            // 0: the gather failed or an earlier error is pending: move nothing
    uint32_t n_u;           // distinct IDs
    uint32_t stamp;         // minibatch index
    uint32_t next_chunk;    // work counter of the row mover's link half (reset by the commit kernel)
};

// One queued row move of the accumulator (Section 3.2: the accesses of several minibatches go out in one
// launch).  A fill crosses the host link; a copy stays in HBM.
struct FillOp {
    const void* src;        // host store row or CPU-buffer row (device-visible address)
    void* dst_out;          // row in a caller's output tensor
    uint64_t dst_line;      // cache line to fill as well, or NO_LINE
    uint32_t late;          // index of the late line fill (a copy output row -> line) this fill owns, or NO_OP
    uint32_t pad;
};
struct CopyOp {
    const void* src;
    void* dst;              // nullptr: cancelled
};

// Mirror of gids_stats in host-mapped memory, written by the finalize kernel.
struct StatsRec {
    uint64_t seq, n_unique, n_hit, n_cpu_hit, n_miss, n_bypass, n_pending;
    int32_t flushed, status;
    uint64_t n_line_fills;
    uint64_t n_cpu_again;
};

// Everything the gather kernels need about one cache.
template <typename IdT>
struct CacheView {
    uint64_t n_rows;        // rows of the store
    uint64_t n_sets;
    uint32_t ways, lg_ways;
    uint32_t row_bytes, line_bytes;
    uint32_t words_per_set; // 64-bit words of the miss mask per set
    uint32_t use32;         // n_rows and n_sets < 2^32: set index with 32-bit arithmetic
    uint32_t rows_per_line; // node rows one cache line holds (store line b = id div rows_per_line is the tag)
    uint32_t policy;        // order of evictable ways: 0 = last-use stamp (LRU by minibatch), 1 = seeded hash (random)
    uint64_t policy_key;    // mix64(seed + 8 * golden): prefix of the random policy's hash chain
    IdT* tags;              // lines, -1 = empty
    int32_t* stamps;        // lines, -1 = never used
    uint32_t* pending;      // lines: index of the queued fill that will write the line (valid while fillgrp == open group)
    uint32_t* fillgrp;      // lines: group in which the line's fill was queued
    uint32_t* hitgrp;       // lines: group in which a copy out of the line was last queued
    uint8_t* reuse;         // n_rows: buffered future minibatches that contain the node
    uint64_t* missmask;     // n_sets * words_per_set
    const uint64_t* hotbits;    // n_rows / 64 words, or nullptr when no CPU buffer
    const uint32_t* hotrank;    // exclusive popcount prefix of hotbits
    char* cache_data;       // lines * line_bytes
    const char* store;      // device-visible address of the host store
    const char* cpubuf;     // device-visible address of the CPU buffer rows (ascending ID order)
    char** cpu_first;       // per CPU-buffer row: the output row the open group's first fill of it writes (or nullptr: not kept)
    Ctl* ctl;
};

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

// set = v mod n_sets, round = v div n_sets (the position of v among the IDs that share its set)
template <typename IdT>
__device__ __forceinline__ void set_and_round(const CacheView<IdT>& c, uint64_t v, uint64_t* set, uint64_t* round) {
    if (c.use32) {
        const uint32_t q = (uint32_t)v / (uint32_t)c.n_sets;
        *round = q;
        *set = (uint32_t)v - q * (uint32_t)c.n_sets;
    } else {
        const uint64_t q = v / c.n_sets;
        *round = q;
        *set = v - q * c.n_sets;
    }
}

// the store line (the cache's tag) that holds row v
template <typename IdT>
__device__ __forceinline__ uint64_t store_line_of(const CacheView<IdT>& c, uint64_t v) {
    if (c.rows_per_line == 1) return v;
    return c.use32 ? (uint64_t)((uint32_t)v / c.rows_per_line) : v / c.rows_per_line;
}

// Device-side counters of the neighbour sampler.
struct SamplerState {
    uint32_t n_raw;         // raw IDs written so far (seeds + every finished hop)
    uint32_t layer_base;    // where the current hop's neighbours start in the raw list
    uint32_t layer_count;   // how many the current hop produced
    uint32_t ticket;
};

// ---- launchers (defined in the .hip files) ---------------------------------

template <typename IdT>
void launch_mark(const IdT* ids, uint64_t n, const uint32_t* n_dev, uint64_t n_rows, uint64_t* bitmap, Ctl* ctl,
                 hipStream_t s);

void launch_count(const uint64_t* bitmap, uint64_t n_words, uint32_t* blocksum, uint32_t* blockoff, Ctl* ctl,
                  uint32_t* n_out, hipStream_t s);

template <typename IdT>
void launch_emit(uint64_t* bitmap, uint64_t n_words, uint64_t n_rows, const uint32_t* blockoff, IdT* dst,
                 uint8_t* reuse_inc, uint32_t* wrank, bool clear, Ctl* ctl, uint32_t* n_out_solo, hipStream_t s);

template <typename IdT>
void launch_verify(const IdT* fresh, const IdT* head, const uint32_t* head_n, Ctl* ctl, uint64_t n_upper,
                   hipStream_t s);

template <typename IdT>
void launch_inverse(const IdT* ids, uint64_t n, const uint64_t* bitmap, const uint32_t* wrank, uint32_t* inverse,
                    Ctl* ctl, hipStream_t s);

template <typename IdT>
void launch_clear(uint64_t* bitmap, const IdT* unique, const uint32_t* n_u, uint64_t n_upper, hipStream_t s);

template <typename IdT>
void launch_probe(const CacheView<IdT>& c, const IdT* unique, const uint32_t* n_u, uint64_t n_upper,
                  uint64_t out_capacity, bool pop_window, uint64_t* plan, hipStream_t s);

template <typename IdT>
void launch_victim(const CacheView<IdT>& c, const IdT* unique, const uint32_t* n_u, uint64_t n_upper,
                   uint64_t* plan, hipStream_t s);

template <typename IdT>
void launch_commit(const CacheView<IdT>& c, const IdT* unique, const uint32_t* n_u, uint64_t n_upper,
                   const uint64_t* plan, BatchHdr* hdr, hipStream_t s);

template <typename IdT>
void launch_move(const CacheView<IdT>& c, const IdT* unique, BatchHdr* hdr, uint64_t n_upper,
                 const uint64_t* plan, char* out, IdT* unique_out, int blocks, int link_blocks_max, hipStream_t s);

// what the accumulator's kernels need besides the cache view
struct AccumView {
    FillOp* fills[2];
    CopyOp* rcopies[2];
    CopyOp* wcopies[2];
    uint64_t cap;           // entries of each list
};

template <typename IdT>
void launch_queue(const CacheView<IdT>& c, const AccumView& a, uint32_t group, const IdT* unique, const BatchHdr* hdr,
                  uint64_t n_upper, const uint64_t* plan, char* out, IdT* unique_out, hipStream_t s);

// commit + (with the accumulator) queueing + header and counters, in one launch
template <typename IdT>
void launch_settle(const CacheView<IdT>& c, const AccumView& a, uint32_t group, int accum, const IdT* unique,
                   const uint32_t* n_u, uint64_t n_upper, const uint64_t* plan, BatchHdr* hdr, char* out,
                   IdT* unique_out, StatsRec* rec, uint64_t seq, hipStream_t s);

// Division of a 32-bit number by a divisor fixed on the host: the quotient is the high half of the product with
// ceil(2^64 / d), exact for every 32-bit dividend (d = 1 is its own case: that multiplier does not fit).
struct FastDiv {
    unsigned long long magic;
    uint32_t d;
};
inline FastDiv make_fast_div(uint32_t d) { return FastDiv{d <= 1 ? 0ull : ~0ull / d + 1, d}; }
__device__ __forceinline__ uint32_t fast_div(const FastDiv& f, uint32_t v) {
    return f.d <= 1 ? v : (uint32_t)__umul64hi((unsigned long long)v, f.magic);
}

// ---- merged iterations: k steps (push one list, gather the window's head) in one call
template <typename IdT>
struct ManyPushes {                     // the lists the call pushes, one workgroup each
    const IdT* ids[MANY_MAX];           // raw list
    uint64_t n[MANY_MAX];
    IdT* dst[MANY_MAX];                 // window slot that receives the ascending distinct IDs
    uint32_t slot[MANY_MAX];            // its entry of Ctl::win_n
};
template <typename IdT>
struct ManySteps {
    uint32_t k;
    uint64_t seq0;                      // gather index of step 0
    const IdT* pushed[MANY_MAX];        // distinct list pushed in step i (nullptr: none), and its count's entry
    uint32_t pushed_slot[MANY_MAX];
    const IdT* head[MANY_MAX];          // distinct list gathered in step i
    uint32_t head_slot[MANY_MAX];
    uint64_t out_capacity[MANY_MAX];
    uint64_t plan_offset[MANY_MAX];     // where step i's plan starts in the call's plan buffer
    char* out[MANY_MAX];
    IdT* unique_out[MANY_MAX];
    // the distinct window slots behind `pushed` and `head` (a list pushed in one step is the head of a later
    // one), so that a workgroup picks the IDs of its own cache sets out of every list once
    uint32_t n_lists;
    const IdT* list[2 * MANY_MAX];
    uint16_t list_slot[2 * MANY_MAX];
    uint8_t list_is_head[2 * MANY_MAX];
    uint8_t head_list[MANY_MAX];        // step i's head, as an index into `list`
    uint8_t pushed_list[MANY_MAX];      // the list pushed in step i (MANY_NO_LIST: none)
    uint32_t share_cap;                 // entries of one list a workgroup can keep (<= its thread count)
    FastDiv div_sets;                   // division by the number of sets
    uint32_t wg_shift;                  // the launch has 2^wg_shift workgroups
    uint32_t resident;                  // the workgroups keep their sets' state in LDS for the length of the kernel
    uint32_t sets_per_wg;               // places for sets in that LDS: ceil(n_sets / workgroups)
    uint32_t rounds;                    // nodes per set: ceil(n_rows / n_sets)
    uint32_t group_dedup;               // a CPU-buffer row that several steps need crosses the link once per call
    // a call whose lists do not fit a workgroup's LDS all at once is classified in several launches, each with the
    // steps [step0, step0 + k) of the call; the group stays open between them
    uint32_t step0;
    uint32_t closes_group;              // this launch holds the call's last step
};
constexpr uint8_t MANY_NO_LIST = 0xFF;
uint64_t many_max_rows();
bool many_fits(uint64_t n_rows, uint64_t n_sets, uint32_t ways, uint32_t words_per_set, size_t id_bytes, uint32_t n_lists,
               uint64_t longest, uint64_t pool_bytes, bool group_dedup, bool* state_in_lds = nullptr);
uint32_t many_max_ways();
template <typename IdT>
void launch_dedup_small(const ManyPushes<IdT>& p, uint32_t n_lists, uint64_t n_rows, Ctl* ctl, hipStream_t s);
template <typename IdT>
void launch_classify_many(const CacheView<IdT>& c, const AccumView& a, uint32_t group, ManySteps<IdT>& m,
                          uint64_t longest, uint64_t pool_bytes, uint64_t* plan_all, StatsRec* ring, uint32_t ring_size,
                          hipStream_t s);   // fills m.share_cap (m.group_dedup: by the caller); pool_bytes = 0: every workgroup reads the lists from memory

// The distinct-ID lists of a group's minibatches wait in a staging buffer of the group (they are produced on
// the stream that classifies) and reach the callers' buffers with the rows, on the stream the callers gave.
struct UniqCopies {
    void* dst[MANY_MAX];            // caller's unique_dev of the i-th minibatch of the group, or nullptr
    uint64_t src_entry[MANY_MAX];   // where its list starts in the staging buffer (entries)
    uint32_t n;                     // minibatches in the group
};

template <typename IdT>
void launch_group_move(const CacheView<IdT>& c, const AccumView& a, uint32_t parity, uint64_t rows_upper,
                       int hbm_blocks_max, int link_blocks_max, const UniqCopies& u, const IdT* stage, hipStream_t s);

uint64_t sampler_key(uint64_t seed, uint64_t tag);
uint64_t sampler_mix(uint64_t z);

template <typename IdT>
void launch_seeds(uint64_t ks, uint64_t n_seeds, uint64_t n_nodes, const uint64_t* rank_table, uint64_t perm_mult,
                  uint64_t perm_add, IdT* raw, SamplerState* st, hipStream_t s);

// one hop: frontier -> neighbours appended to raw[] and written to hop_out[] (the next frontier's input)
template <typename IdT>
void launch_hop(const IdT* frontier, const uint32_t* n_front, uint64_t front_upper, const int64_t* indptr,
                const IdT* indices, uint32_t fanout, uint64_t kl, uint32_t* blocksum, uint32_t* blockoff, IdT* raw,
                IdT* hop_out, SamplerState* st, hipStream_t s);

// expected visits per node under the sampler's law; cur / nxt are n-entry scratch arrays
template <typename IdT>
void launch_visit_scores(const int64_t* indptr, const IdT* indices, uint64_t n, const uint32_t* fanouts,
                         uint32_t n_layers, uint64_t n_seeds, uint64_t* cur, uint64_t* nxt, uint64_t* score,
                         hipStream_t s);

// weighted reverse PageRank after n_iters power iterations; scratch is an n-entry array
template <typename IdT>
void launch_reverse_pagerank(const int64_t* indptr, const IdT* indices, uint64_t n, uint32_t damping_q16,
                             uint32_t n_iters, uint64_t* scratch, uint64_t* score, hipStream_t s);

void launch_calibrate(const char* store, uint64_t store_rows, uint32_t row_bytes, char* out, uint32_t n,
                      hipStream_t s);

// accum: 0 = no accumulator, 1 = this gather leaves its rows queued, 2 = this gather closes its group
void launch_finalize(Ctl* ctl, StatsRec* rec, uint64_t seq, const uint32_t* n_u, int accum, hipStream_t s);

void launch_fill_u32(uint32_t* p, uint64_t n, uint32_t value, hipStream_t s);
void launch_fill_i64(int64_t* p, uint64_t n, int64_t value, hipStream_t s);

}  // namespace gids
