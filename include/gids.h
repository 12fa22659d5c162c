/* gids.h - C ABI of the MI355X minibatch feature-gather library (libgids.so).
 *
 * The library implements the feature-aggregation ("gather") stage of a GNN
 * dataloader as the GIDS paper (arxiv 2306.16384) poses it: the node IDs a
 * neighbourhood sampler produced for one minibatch are deduplicated, and the
 * feature row of every distinct ID is fetched into a minibatch buffer in GPU
 * memory (Section 2.2.3), looking first in a set-associative software cache in
 * GPU memory whose eviction is steered by a window of future minibatches
 * (Section 3.4), then in a constant buffer of hot rows pinned in CPU memory
 * (Section 3.3), then in the backing feature store.  The backing store here is
 * a host-pinned buffer that kernels read zero-copy over the host link; it
 * stands in for the paper's SSDs.  Fills from the store can be batched across
 * minibatches by an accumulator (Section 3.2).
 *
 * Conventions
 *   - Every function returns 0 (GIDS_OK) or a negative GIDS_E_* code;
 *     gids_last_error() returns a thread-local text for the last failure.
 *   - Handles are opaque and owned by the library.  Every buffer named in an
 *     argument is owned by the caller.  "dev" = device (HBM) pointer, "host" =
 *     ordinary host pointer unless stated otherwise.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls that take a stream only enqueue work and return; they never block
 *     on the device unless an internal buffer has to grow (avoid that with
 *     gids_cache_reserve).  Inputs are read, and outputs are complete, in the
 *     order of the stream given to the call.  For caches of 32 MiB and more the
 *     library runs dedup, probe and victim selection on a stream of its own
 *     and orders it against the caller's streams with events, so that the
 *     classification of one minibatch overlaps the row movement of the
 *     previous one (of the previous group, with the accumulator); to let it
 *     overlap, give gids_window_push a different stream (the one the sampler
 *     fills ID lists on) than gids_gather (the one that consumes the rows).
 *     All gathers of one cache use one stream, all pushes one stream (the same
 *     or another).
 *   - Threads: calls on one cache (or one graph) must not overlap in time;
 *     the caller serialises them.  Different caches, graphs and stores may be
 *     used from different threads at once, and several caches may share one
 *     store (it is only read).  A store must outlive the caches created on it.
 *     The library works on the device that is current when the store is
 *     created; keep that device current for every later call.
 *   - IDs are signed integers of the width fixed at store creation (4 or 8
 *     bytes), valid range [0, n_rows).
 *   - Errors found by the device (an ID out of range, a gather that does not
 *     match the buffered window head, an output buffer too small) cannot be
 *     returned by the enqueueing call.  The failing operation changes nothing,
 *     the error is recorded in that minibatch's gids_stats.status, and it is
 *     sticky: once the host has seen it (gids_stats_read, or any later
 *     push, gather or flush called after the failing gather finished) every
 *     later call on the cache returns it.  A HIP runtime failure in the middle
 *     of a push or gather closes the cache the same way (GIDS_E_HIP).
 */
#ifndef GIDS_H
#define GIDS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GIDS_OK 0
#define GIDS_E_INVAL (-1) /* bad argument or call out of protocol            */
#define GIDS_E_NOMEM (-2) /* host or device allocation failed                */
#define GIDS_E_RANGE (-3) /* a node ID outside [0, n_rows)                   */
#define GIDS_E_ORDER (-4) /* gather does not match the head of the window    */
#define GIDS_E_FULL (-5)  /* window already holds window_depth + 1 lists     */
#define GIDS_E_HIP (-6)   /* HIP runtime error, text in gids_last_error()    */
#define GIDS_E_SPACE (-7) /* caller's output buffer has too few rows         */

typedef struct gids_store gids_store;
typedef struct gids_cache gids_cache;

/* Per-minibatch counters (the paper's reported quantity is the hit ratio,
 * Section 4.5).  n_hit + n_cpu_hit + n_miss == n_unique.  n_bypass (a subset of
 * n_miss) counts misses that found no evictable line and were served from the
 * store without being installed.  With the accumulator, n_pending = rows (of
 * this and earlier minibatches) still queued in the open group when the gather
 * call's own work ends, and `flushed` is 1 when this gather closed its group,
 * i.e. when every row of its output and of the earlier queued ones has been
 * written by then; without it they are 0 and 1.  n_line_fills = cache
 * lines this minibatch fills from the store: n_miss - n_bypass with one row
 * per line, fewer when several missing rows share a line.  n_cpu_again (a
 * subset of n_cpu_hit; 0 unless gids_cache_set_group_dedup is on) counts the
 * CPU-buffer rows that an earlier minibatch of the same group already brings
 * over the link and that this minibatch receives as a copy inside device
 * memory. */
typedef struct gids_stats {
    uint64_t seq;       /* 0-based index of the gather call on this cache */
    uint64_t n_unique;
    uint64_t n_hit;
    uint64_t n_cpu_hit;
    uint64_t n_miss;
    uint64_t n_bypass;
    uint64_t n_pending;
    int32_t flushed;
    int32_t status;     /* GIDS_OK or the GIDS_E_* the device found */
    uint64_t n_line_fills;
    uint64_t n_cpu_again;
} gids_stats;

/* The feature table (Section 2.1: an N x D matrix, one row per node).
 * n_rows x row_bytes bytes in pinned host memory that the GPU reads zero-copy.
 * row_bytes must be a multiple of 16.  id_bytes is 4 or 8.
 * host_ptr_or_null: NULL - the library allocates pinned memory (free with
 * gids_store_destroy; fill it through gids_store_host_ptr before the first
 * gather); otherwise memory the caller already allocated with hipHostMalloc
 * (e.g. a pinned torch tensor) holding the table, which must outlive the store.
 * Ordinary pageable memory is rejected with GIDS_E_HIP. */
int gids_store_create(uint64_t n_rows, uint32_t row_bytes, uint32_t id_bytes, void* host_ptr_or_null,
                      gids_store** out);
void* gids_store_host_ptr(gids_store* store);
int gids_store_destroy(gids_store* store);

/* Measure the store as the row mover sees it, for Eq. 2-3 of Section 3.2: the
 * library times two copies of hashed rows (2,048 and 65,536 of them) from the
 * host table to a scratch buffer and fits time = overhead + rows / rate.
 * *rows_per_s plays the role of IOPS_peak, *overhead_s that of the initial plus
 * termination latency: gids_accum_threshold(rows_per_s, overhead_s, 0, r, 1) is
 * then the number of rows a minibatch (or an accumulated group of minibatches)
 * must send over the link to keep it at the fraction r of its peak.  Blocks;
 * the table need not be filled. */
int gids_store_calibrate(gids_store* store, double* rows_per_s, double* overhead_s);

/* The GPU software cache over a store (Section 3.4) plus its window buffer
 * and fill accumulator (Section 3.2).
 *   lines          cache lines, a multiple of `ways`; one node row per line
 *                  unless gids_cache_set_rows_per_line says otherwise
 *   ways           associativity, a power of two in [1, 64]; set = id mod (lines / ways)
 *   line_bytes     slot stride in HBM, >= row_bytes, multiple of 16
 *   window_depth   W in [0, 254]: how many minibatches beyond the one being
 *                  gathered are buffered.  A cached row that one of them reuses
 *                  is not evicted.  W = 0: no window, plain LRU by minibatch
 *                  (or the policy set with gids_cache_set_policy).
 *   accum_threshold  0: every gather moves its own rows before it ends.
 *                  > 0: the storage access accumulator of Section 3.2.
 *                  Consecutive gathers are merged into a group until the node
 *                  accesses they bring (entries of their raw ID lists) reach
 *                  this number; a gather only classifies its minibatch and
 *                  queues its rows, and when the group closes the rows of all
 *                  its minibatches move in one launch (two, when some copies
 *                  depend on others).  A group also closes after
 *                  GIDS_ACCUM_MAX_MERGE gathers and at gids_flush.  The
 *                  counters and the final contents of every output are the
 *                  same for any threshold; what changes is when an output is
 *                  complete (gids_stats.flushed, gids_flush).  See
 *                  gids_cache_set_accum_mode for the adaptive threshold.
 * Device memory taken: lines * line_bytes for the data plus about
 * 12-16 bytes per line, n_rows / 8 * 3 bytes of bitmaps and n_rows bytes of
 * reuse counters. */
int gids_cache_create(gids_store* store, uint64_t lines, uint32_t ways, uint32_t line_bytes,
                      uint32_t window_depth, uint64_t accum_threshold, gids_cache** out);
int gids_cache_destroy(gids_cache* cache);

/* How the accumulator's threshold is read (call before the first gather).
 * GIDS_ACCUM_FIXED (default): accum_threshold counts node accesses.
 * GIDS_ACCUM_ADAPTIVE: accum_threshold is the number of accesses that should
 * reach the backing store per launch (N of Eq. 2-3, see gids_accum_threshold
 * and gids_store_calibrate), and the library raises the node-access threshold
 * by the share of accesses that the GPU cache and the CPU buffer take away
 * (Section 3.2, last paragraph): with A node accesses and S store accesses
 * (misses) counted over every gather at least GIDS_ACCUM_LAG calls back,
 *   threshold = clamp(ceil(accum_threshold * A / S), accum_threshold,
 *                     GIDS_ACCUM_MAX_RAISE * accum_threshold)
 * (accum_threshold while A == 0, the upper bound while S == 0).  The fixed lag
 * makes the grouping a pure function of the ID lists; a gather call waits for
 * the counters of the gather GIDS_ACCUM_LAG + 1 calls back if the device has
 * not produced them yet.  For lists pushed with gids_window_push_dev a node
 * access count is the list's n_max. */
#define GIDS_ACCUM_FIXED 0
#define GIDS_ACCUM_ADAPTIVE 1
#define GIDS_ACCUM_MAX_MERGE 32
#define GIDS_ACCUM_LAG 16
#define GIDS_ACCUM_MAX_RAISE 8
int gids_cache_set_accum_mode(gids_cache* cache, int mode);

/* Section 3.2 merges the accesses of consecutive iterations; merged, accesses to
 * the same row of the constant CPU buffer (Section 3.3) can be served by one
 * transfer.  on != 0: within one group of minibatches (a gids_gather_many call,
 * or the gathers that accum_threshold puts into one group) a CPU-buffer row
 * that several of them need crosses the host link once, for the first of
 * them, and reaches the others' outputs as a copy of that output row inside
 * device memory (with the group's other dependent copies, after its fills).
 * Outputs and counters are the same either way (n_cpu_hit counts every access,
 * n_cpu_again those served by a copy); what changes is the traffic over the
 * link.  Off by default: the per-minibatch cost model of the measurements
 * charges every CPU-buffer hit one row over the link.  Needs a cache created
 * with accum_threshold > 0; not while a group of minibatches is open
 * (GIDS_E_INVAL). */
int gids_cache_set_group_dedup(gids_cache* cache, int on);

/* Base replacement policy, i.e. the order in which the evictable ways of a set
 * are given to misses (window pinning applies to both; call before the first
 * gather).  GIDS_POLICY_LRU (default): least recently used by minibatch, ties
 * to the lowest way.  GIDS_POLICY_RANDOM: the policy of the cache the paper
 * builds on (Section 3.4; its window-depth-0 baseline, Section 4.5), made
 * reproducible: empty ways first, then occupied ways in the order of the hash
 * H(seed, 8, minibatch, set, way) (H as in gids_sample). */
#define GIDS_POLICY_LRU 0
#define GIDS_POLICY_RANDOM 1
int gids_cache_set_policy(gids_cache* cache, int policy, uint64_t seed);

/* Cache lines that hold several node rows.  The cache the paper builds on keeps
 * the storage's cache-lines (4 KB in the example of Section 3.3) while a node's
 * row is 512 B to 4 KB (Section 2.1): with small rows one line holds `rows`
 * consecutive rows of the table, and a miss on any of them brings the whole
 * line in, so that its neighbours hit afterwards.  The tag of a line is then
 * the store line number id div rows, its set that number mod (lines / ways);
 * a line stays while any of its rows has a buffered future use.  Every
 * requested row of a missing line counts as a miss of its own (its bytes come
 * from the store); the line is filled once.  rows * row_bytes <= line_bytes;
 * not together with accum_threshold > 0; before the first push or gather.
 * Default 1. */
int gids_cache_set_rows_per_line(gids_cache* cache, uint32_t rows);

/* Pre-size the internal per-minibatch buffers for ID lists of up to
 * max_ids_per_minibatch entries, so that no later call allocates. */
int gids_cache_reserve(gids_cache* cache, uint64_t max_ids_per_minibatch);

/* Constant CPU buffer (Section 3.3): copy the rows of `ids_host` (n distinct
 * IDs, any order) from the store into a second pinned host buffer.  From then
 * on these IDs are served from it and never enter the GPU cache.  Call once,
 * before the first push or gather. */
int gids_cpu_buffer_pin(gids_cache* cache, const void* ids_host, uint64_t n);

/* Window buffer (Section 3.4, Fig. 6 steps 1-4): append the raw ID list
 * (duplicates allowed) of a future minibatch.  Lists are gathered in push
 * order.  GIDS_E_FULL when window_depth + 1 lists are already buffered.
 * With window_depth == 0 that is one list, the next gather's own: it protects
 * nothing from eviction and only lets its deduplication run ahead of the
 * gather call (the gather then takes the pushed list like any window head).
 * To overlap classification with the row movement of earlier gathers, push on
 * another stream than the one that gathers, and keep that stream for the life
 * of the process: HIP multiplexes streams onto a few hardware queues
 * (GPU_MAX_HW_QUEUES, 4 by default) in creation order, and the ordering
 * markers of a push stream that shares the gather stream's queue wait behind
 * the row mover, which serialises the two (results stay correct). */
int gids_window_push(gids_cache* cache, const void* ids_dev, uint64_t n, void* stream);

/* The same with the list's length in device memory (*n_dev <= n_max entries of
 * ids_dev are valid): for ID lists a GPU sampler produced, whose length the host
 * never learns.  n_max bounds the work and sizes the window slot. */
int gids_window_push_dev(gids_cache* cache, const void* ids_dev, uint64_t n_max, const uint32_t* n_dev, void* stream);

/* Gather one minibatch: feature aggregation as Section 2.2.3 defines it (the
 * feature rows of the sampled nodes, collected into one minibatch buffer in
 * GPU memory), served through the cache of Section 3.4 and the CPU buffer of
 * Section 3.3.
 *   ids_dev, n       the raw ID list.  When a list is buffered (always the
 *                    case with window_depth > 0; after a push with
 *                    window_depth == 0) it must have the same distinct IDs as
 *                    the oldest buffered list (else GIDS_E_ORDER in stats), or
 *                    be NULL (n ignored) to gather that list as it was pushed.
 *   out_dev          receives row j = feature row of the j-th smallest distinct
 *                    ID, rows packed at row_bytes; out_capacity_rows rows are
 *                    available (GIDS_E_SPACE in stats when there are more
 *                    distinct IDs; n rows always suffice)
 *   unique_dev       NULL, or room for min(n, out_capacity_rows) IDs (with
 *                    ids_dev == NULL: out_capacity_rows IDs): receives the
 *                    distinct IDs, ascending
 *   inverse_dev      NULL, or n uint32: inverse_dev[i] = j with
 *                    unique[j] == ids_dev[i] (requires ids_dev)
 * With accum_threshold > 0 the output buffers (out_dev, unique_dev) of gathers
 * whose group has not closed must stay untouched until it has (stats.flushed
 * of a later gather / gids_flush); they are complete in stream order after
 * the call that closes the group. */
int gids_gather(gids_cache* cache, const void* ids_dev, uint64_t n, void* out_dev, uint64_t out_capacity_rows,
                void* unique_dev, void* inverse_dev, void* stream);

/* The same gather for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * gids_gather keeps its per-minibatch buffers (plan, ID scratch, headers) in
 * device memory it sizes on demand; this entry point keeps them in a fixed
 * array inside the library instead (32 MiB + 256 B per GPU, held from the
 * moment the library is loaded on that GPU until the process ends) and calls no
 * allocating routine.  Arguments and results are those of gids_gather without
 * the inverse map.  Limits: the raw list (and, when a buffered list is gathered,
 * the list that was pushed) has at most GIDS_STATIC_MAX_IDS entries, else
 * GIDS_E_INVAL; not on a cache with accum_threshold > 0 (its queues grow on
 * demand).  Lists a window buffers are still stored by gids_window_push, which
 * allocates when a list is longer than any before: call gids_cache_reserve
 * first.  Every call on a GPU, from whichever cache, shares the one array, and
 * the array keeps the last call's contents (nothing in it has to start at
 * zero: each call writes every entry it reads): calls on one cache order
 * themselves like gids_gather's and may be mixed with them, but calls on
 * different caches of one GPU race unless the stream of the earlier one has
 * been synchronised before the later one is made. */
#define GIDS_STATIC_MAX_IDS (1u << 20)
int gids_gather_static(gids_cache* cache, const void* ids_dev, uint64_t n, void* out_dev, uint64_t out_capacity_rows,
                       void* unique_dev, void* stream);

/* Merged iterations (Section 3.2: the data preparation of consecutive
 * iterations is merged, which takes the stop-and-go boundaries between
 * minibatches away).  One call brings k steps of the steady-state loop,
 *   step i:  gids_window_push(push_ids_dev[i], push_n[i])   if push_ids_dev[i] != NULL
 *            gids_gather(NULL, 0, out_dev[i], out_capacity_rows[i], unique_dev[i], NULL)
 * with exactly the results of those calls made one after the other (outputs,
 * counters, cache state), and runs them as ONE accumulator group whatever the
 * cache's accum_threshold says: a group that is open when the call arrives is
 * closed first, the call's own group closes with its last step (gids_stats of
 * step i: n_pending = rows of steps 0..i, flushed = 0; the last step: 0 and 1).
 * Every output of the call is complete, in stream order, when the call's work
 * ends.  With ways <= 16, one row per line and LDS room for a workgroup's share
 * of every list of the call (lists of tens of thousands of distinct IDs at
 * k = 32, of more than a hundred thousand at k <= 16; where the sets' state is
 * in device memory anyway a longer call is classified 16, 8 or 4 steps per
 * launch), the k steps take a fixed number of launches: one that deduplicates the pushed lists (a workgroup and
 * an LDS bitmap each; on tables beyond 1.3 M rows three launches per list
 * through the bitmap in device memory), one that classifies the k minibatches
 * one after the other, each workgroup for its own share of the cache sets and,
 * where it fits, with that share's state in its LDS, and the group mover's
 * two.  Other caches and calls take the per-step kernels, still as one group;
 * gids_cache_many_calls tells which way the calls of a cache went.
 * Calls of two steps and more classify on the library's internal stream
 * whatever the cache size (see `push_stream`).
 *   k              1 .. 32 (GIDS_ACCUM_MAX_MERGE)
 *   push_ids_dev   NULL (no step pushes), or k pointers, NULL where a step
 *                  pushes nothing; push_n the lists' lengths
 *   unique_dev     NULL, or k pointers (NULL entries allowed)
 *   push_stream    the stream in whose order the pushed ID lists are ready (and
 *                  may be reused afterwards), as for gids_window_push; `stream`
 *                  the one in whose order the outputs are complete, as for
 *                  gids_gather.  They may be the same; with two, the
 *                  classification of one call overlaps the row movement of the
 *                  call before
 * Needs a cache created with accum_threshold > 0 (it owns the group lists);
 * errors as gids_window_push / gids_gather; a device-found error in step i
 * leaves steps i.. undone and is reported in their gids_stats.status. */
int gids_gather_many(gids_cache* cache, uint32_t k, const void* const* push_ids_dev, const uint64_t* push_n,
                     void* const* out_dev, const uint64_t* out_capacity_rows, void* const* unique_dev, void* push_stream,
                     void* stream);

/* The accumulator's forced launch (Section 3.2: accesses merged over several
 * minibatches go out in one launch; this is the launch without waiting for
 * the threshold).  Moves every queued row now: after the stream reaches the
 * end of this call's work the output of every earlier gather is complete.
 * Does not block.  Returns the error of an earlier gather if the device has
 * reported one by now (the rows of a failed gather are never moved). */
int gids_flush(gids_cache* cache, void* stream);

/* Hit, CPU-buffer and miss counts per minibatch (the quantities behind the
 * hit ratios of Section 4.5 and the redirected share of Section 4.4).
 * Waits for gather number `seq` (0-based) to finish on the device and returns
 * its counters.  Only the most recent 64 gathers are kept.  Returns
 * stats->status. */
int gids_stats_read(gids_cache* cache, uint64_t seq, gids_stats* stats);

/* Number of gathers enqueued so far (the next gather's seq). */
uint64_t gids_cache_gathers(const gids_cache* cache);

/* How the gids_gather_many calls of this cache were carried out so far: calls
 * that ran through the merged kernels, calls that took the per-step kernels
 * as one group (see gids_gather_many for what decides).  Either may be NULL. */
void gids_cache_many_calls(const gids_cache* cache, uint64_t* merged_kernels, uint64_t* per_step_kernels);

/* Inspection for tests and tools: blocks until the stream is idle, then copies
 * the tag (int64, -1 = empty) and last-use stamp (int64, -1 = never) of every
 * line to host arrays of `lines` entries each.  Either may be NULL. */
int gids_cache_snapshot(gids_cache* cache, int64_t* tags_host, int64_t* stamps_host);

/* Per-phase device time of each gather, for benchmarks and profiling.  When
 * enabled, gids_gather records HIP events around its three phases, each pair
 * on the stream the phase's kernels are launched on; gids_profile_read waits
 * for gather `seq` and writes milliseconds to ms3: [0] ID dedup/sort (+ window
 * check, inverse map), [1] CPU-buffer lookup + tag probe + victim selection +
 * commit + counters, [2] row movement (hit scatter, line fills, CPU-buffer
 * rows; the accumulator's queueing and flush when accum_threshold > 0).
 * Phases of consecutive gathers overlap, so the three do not add up to the
 * step time.  Off by default. */
int gids_profile_enable(gids_cache* cache, int on);
int gids_profile_read(gids_cache* cache, uint64_t seq, float* ms3);

/* ---- GPU neighbourhood sampler (the stage before the gather) ----------------
 * Graph structure in CSR form for sampling by GPU threads (Section 3.5: the
 * structure data is a few percent of the dataset and is kept out of storage).
 *   indptr_host    n_nodes + 1 int64, indptr[0] == 0
 *   indices_host   indptr[n_nodes] neighbour IDs of id_bytes each
 *   zero_copy      0: both arrays are copied into GPU memory (they may be freed
 *                  after the call); 1: they stay where they are and are read
 *                  zero-copy, as in the paper - they must then be hipHostMalloc
 *                  memory that outlives the graph */
typedef struct gids_graph gids_graph;
int gids_graph_create(uint64_t n_nodes, const int64_t* indptr_host, const void* indices_host, uint32_t id_bytes,
                      int zero_copy, gids_graph** out);
int gids_graph_destroy(gids_graph* graph);

/* Largest raw list a minibatch can have: n_seeds * (1 + f0 + f0*f1 + ...). */
uint64_t gids_sample_capacity(const uint32_t* fanouts_host, uint32_t n_layers, uint64_t n_seeds);

/* Sample minibatch number `batch` (Section 2.2.2: up to fanout neighbours per
 * node per layer, uniformly at random, without replacement; each hop expands
 * the distinct nodes the previous hop reached).  Every draw is a counter-based
 * hash of (seed, batch, layer, node, draw), so the list is a pure function of
 * the arguments: seed node i = H(seed, 4, batch, i) mod n_nodes, or, with a
 * rank table (n_nodes ascending uint64 thresholds, CDF scaled to 2^63, in
 * device memory), rank = #{thresholds <= H >> 1} mapped to node
 * (rank * perm_mult + perm_add) mod n_nodes; a node of degree d > fanout f gets
 * f distinct adjacency slots by Floyd's subset sampling with draws
 * H(seed, 5, batch, layer, node, j) mod (j + 1), j = d-f .. d-1.  H chains the
 * SplitMix64 output function; the formulas are spelled out in csrc/sampler.hip.
 *   raw_dev        receives the seeds, then each hop's neighbours in (node
 *                  ascending, draw) order, duplicates kept; raw_capacity must
 *                  be >= gids_sample_capacity(...) (else GIDS_E_SPACE)
 *   n_raw_dev      device uint32: receives the list's length
 * Feed the result to gids_window_push_dev / gids_gather.  Calls on one graph
 * must be ordered by the caller (one stream). */
int gids_sample(gids_graph* graph, uint64_t seed, uint64_t batch, const uint32_t* fanouts_host, uint32_t n_layers,
                uint64_t n_seeds, const uint64_t* rank_table_dev, uint64_t perm_mult, uint64_t perm_add, void* raw_dev,
                uint64_t raw_capacity, uint32_t* n_raw_dev, void* stream);

/* Hot-node ranking for gids_cpu_buffer_pin (Section 3.3 ranks nodes by a
 * weighted reverse PageRank that estimates how often sampling reaches them;
 * the paper gives no formula, this is the exact expectation for gids_sample's
 * law with uniform seeds, ignoring only that a hop's frontier is deduplicated
 * beyond clamping each node's expected presence at 1).
 * scores_dev receives n_nodes uint64 in 32.32 fixed point: the expected number
 * of times each node appears in a minibatch's raw list,
 *   lam_0(v) = n_seeds / n;  lam_(l+1)(u) = sum over adjacency slots v -> u of
 *   min(1, lam_l(v)) * min(deg v, f_l) / deg v;  score = lam_0 + ... + lam_L,
 * every product and quotient in integers (floor), so the result is exact and
 * reproducible.  Blocks until done (a set-up step, not part of the hot path). */
int gids_graph_visit_scores(gids_graph* graph, const uint32_t* fanouts_host, uint32_t n_layers, uint64_t n_seeds,
                            uint64_t* scores_dev, void* stream);

/* The hot-node metric Section 3.3 names: weighted reverse PageRank.  Rank
 * flows along the adjacency slots (the way sampling walks, against the
 * direction of the dataset's edges), a node of degree deg passing 1/deg of its
 * damped rank along each slot; uniform teleport; nodes without slots pass
 * nothing on.  Power iteration in integers with total mass 2^44:
 *   base = floor(2^44 / n);  r_0 = base;  teleport = floor(base * (65536 - damping_q16) / 65536)
 *   r_(k+1)(u) = teleport + sum over slots v -> u of floor(floor(r_k(v) * damping_q16 / 65536) / deg v)
 * scores_dev receives r_(n_iters) as n_nodes uint64 (device).  damping_q16 in
 * [0, 65536], n_iters <= 10000, else GIDS_E_INVAL.  Blocks until done (a
 * set-up step, not part of the hot path). */
int gids_graph_reverse_pagerank(gids_graph* graph, uint32_t damping_q16, uint32_t n_iters, uint64_t* scores_dev,
                                void* stream);

/* Number of in-flight fills an accumulator needs so that a storage device of
 * `iops_peak` requests/s per device sustains `ratio` of its peak, given the
 * latency of the initial and termination phases in seconds (Section 3.2,
 * Eq. 2-3).  Pure host arithmetic; a helper for choosing accum_threshold. */
double gids_accum_threshold(double iops_peak, double t_initial, double t_termination, double ratio, int n_ssd);

const char* gids_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* GIDS_H */
