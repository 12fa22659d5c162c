// The C ABI of libgids.so (declared in include/gids.h): argument checks, buffer
// ownership, the window FIFO and the order in which the kernels of one push or
// gather are enqueued.  No step of the gather itself runs on the host.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "../../include/gids.h"
#include "gids_dev.h"

namespace gids {
uint32_t scan_blocks(uint64_t n_words);
}  // namespace gids

using namespace gids;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(expr)                                                                           \
    do {                                                                                        \
        hipError_t e_ = (expr);                                                                 \
        if (e_ != hipSuccess) {                                                                 \
            (void)hipGetLastError();                                                            \
            return fail(e_ == hipErrorOutOfMemory ? GIDS_E_NOMEM : GIDS_E_HIP, "%s: %s", #expr, \
                        hipGetErrorString(e_));                                                 \
        }                                                                                       \
    } while (0)

constexpr int STATS_RING = 64;
constexpr uint32_t ACCUM_MAX_MERGE = GIDS_ACCUM_MAX_MERGE;
constexpr uint32_t ACCUM_LAG = GIDS_ACCUM_LAG;
constexpr uint64_t ACCUM_MAX_RAISE = GIDS_ACCUM_MAX_RAISE;
static_assert(GIDS_ACCUM_LAG < STATS_RING, "the adaptive threshold reads counters that must still be in the ring");

// Workspace of gids_gather_static, the gather for callers that must not allocate: what gids_gather keeps in
// buffers it sizes with hipMalloc (the two gather headers, and per parity the plan and the ID scratch, laid out
// for 8-byte IDs) lives in this array instead.  Each GPU holds its own copy at its own address; host code uses
// the address hipGetSymbolAddress returned for the device, never the array's name.
constexpr uint64_t STATIC_MAX_IDS = GIDS_STATIC_MAX_IDS;
constexpr uint64_t STATIC_HDR_BYTES = 256;
constexpr uint64_t STATIC_BYTES = STATIC_HDR_BYTES + 4 * STATIC_MAX_IDS * sizeof(uint64_t);
static __device__ __align__(256) unsigned char scratch[STATIC_BYTES];

constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES] = {};
std::mutex g_scratch_mutex;

// address of `scratch` on the current device (looked up once per device, with that device current)
int static_workspace(int device, void** out) {
    if (device < 0 || device >= MAX_DEVICES) return GIDS_E_INVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            return GIDS_E_HIP;
        }
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return GIDS_OK;
}

bool on_device(int device) {
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return cur == device;
}

template <typename T>
int dev_alloc(T** p, uint64_t count) {
    *p = nullptr;
    if (count == 0) count = 1;
    HIP_TRY(hipMalloc(reinterpret_cast<void**>(p), count * sizeof(T)));
    return GIDS_OK;
}

template <typename T>
void dev_free(T*& p) {
    if (p) (void)hipFree(p);
    p = nullptr;
}

}  // namespace

struct gids_store {
    uint64_t n_rows = 0;
    uint32_t row_bytes = 0, id_bytes = 0;
    void* host = nullptr;   // host address of the table
    void* dev = nullptr;    // the same memory as the GPU sees it
    bool owned = false;
    int device = 0;         // the device that was current when the store was created
};

struct WindowSlot {
    void* ids = nullptr;    // distinct IDs, ascending (device)
    uint64_t cap = 0;       // entries allocated
    uint64_t n_raw = 0;     // length of the raw list that was pushed (bounds the distinct count)
    int64_t last_reader = -1;   // seq of the gather whose row mover read this list last
};

struct gids_cache {
    virtual ~gids_cache() {}
    virtual int init() = 0;
    virtual int reserve(uint64_t n) = 0;
    virtual int pin(const void* ids_host, uint64_t n) = 0;
    virtual int push(const void* ids, uint64_t n, const uint32_t* n_dev, hipStream_t s) = 0;
    virtual int gather(const void* ids, uint64_t n, void* out, uint64_t out_cap, void* unique, void* inverse,
                       bool no_alloc, hipStream_t s) = 0;
    virtual int flush(hipStream_t s) = 0;
    virtual int gather_many(uint32_t k, const void* const* push_ids, const uint64_t* push_n, void* const* outs,
                            const uint64_t* caps, void* const* uniques, hipStream_t ps, hipStream_t s) = 0;
    virtual int snapshot(int64_t* tags, int64_t* stamps) = 0;
    virtual uint32_t window_count() const = 0;

    gids_store* store = nullptr;
    uint64_t lines = 0, n_sets = 0, threshold = 0, n_words = 0;
    uint32_t ways = 0, lg_ways = 0, line_bytes = 0, window = 0, words_per_set = 0;
    int sticky = GIDS_OK;
    uint64_t seq = 0;
    uint64_t many_fast_calls = 0, many_slow_calls = 0;   // gids_gather_many: through the merged kernels / the per-step ones
    uint32_t policy = 0;            // GIDS_POLICY_*
    uint32_t rows_per_line = 1;     // node rows one cache line holds
    uint64_t policy_key = 0;
    void* static_ws = nullptr;      // this device's copy of the static workspace (gids_gather_static)
    // Accumulator (accum_threshold > 0): the host merges consecutive gathers into groups by the node accesses
    // (raw list entries) they bring; the rows of a group move when it closes.
    int accum_mode = GIDS_ACCUM_FIXED;
    int group_override = 0;         // inside a merged call: 1 = this gather keeps its group open, 2 = it closes it
    uint32_t group = 0;             // index of the open group (its lists live in the buffers of parity group & 1)
    uint64_t open_nodes = 0;        // node accesses merged into the open group so far
    uint64_t open_upper = 0;        // bound on the rows queued in the open group
    uint32_t open_batches = 0;
    uint64_t adapt_nodes = 0;       // adaptive mode: node accesses and store accesses of gathers [0, adapt_next)
    uint64_t adapt_store = 0;
    uint64_t adapt_next = 0;
    uint32_t raw_of[STATS_RING] = {};        // raw list length of gather seq, by seq % STATS_RING
    hipEvent_t ev_flush[2] = {};             // the group mover of the last group of each parity has finished
    bool flush_recorded[2] = {false, false};
    StatsRec* ring_host = nullptr;
    StatsRec* ring_dev = nullptr;
    hipEvent_t events[STATS_RING] = {};       // gather seq: its rows have moved (recorded on the caller's stream)
    hipEvent_t ev_meta[STATS_RING] = {};      // gather seq: its metadata kernels and counters are done
    int ev_of[STATS_RING] = {};               // ring entry whose events cover gather seq (a merged call records one pair)
    hipEvent_t ev_hop[16] = {};               // short-lived cross-stream edges
    uint32_t hop = 0;
    // With accum_threshold == 0 the metadata kernels (dedup, probe, victim, commit, counters) run on an
    // internal stream so that they overlap the row movement of earlier gathers on the caller's stream.
    hipStream_t meta = nullptr;
    bool pipelined = false;
    hipStream_t last_stream = nullptr;
    bool have_last = false;
    bool one_stream_work = true;    // a call has queued kernels outside the internal stream since that was last brought up to date
    // Without the internal stream every kernel runs on the stream of its call: a call on another stream
    // than the previous one is ordered after it.
    int follow(hipStream_t s) {
        int rc = GIDS_OK;
        if (!pipelined && have_last && s != last_stream) rc = edge(last_stream, s);
        last_stream = s;
        have_last = true;
        one_stream_work = true;
        return rc;
    }
    // stream `to` waits for everything enqueued on `from` so far
    int edge(hipStream_t from, hipStream_t to) {
        hipEvent_t e = ev_hop[hop++ % 16];
        HIP_TRY(hipEventRecord(e, from));
        HIP_TRY(hipStreamWaitEvent(to, e, 0));
        return GIDS_OK;
    }
    // Distinct IDs per raw ID in the lists of this stream: the largest ratio among the newest finished gathers
    // (1 until one has finished, and approached from there).  Sizes the merged classification, which the host must launch knowing raw
    // lengths only.
    double distinct_ratio = 1.0;
    void update_distinct_ratio() {
        if (!ring_host) return;
        double best = 0.0;
        int seen = 0;
        for (uint64_t g = seq; g-- > 0 && seq - g <= (uint64_t)STATS_RING && seen < 16;) {
            const int r = (int)(g % STATS_RING);
            const StatsRec& rec = ring_host[r];
            if (*reinterpret_cast<const volatile uint64_t*>(&rec.seq) != g) continue;   // not finished yet
            std::atomic_thread_fence(std::memory_order_acquire);  // the record's fields were written before its seq
            if (raw_of[r] == 0 || rec.status) continue;
            best = std::max(best, (double)rec.n_unique / (double)raw_of[r]);
            seen++;
        }
        // (falls by three tenths per call at most: a few lists of many repeats do not undersize the calls after them)
        if (seen) distinct_ratio = std::min(1.0, std::max(best, 0.7 * distinct_ratio));
    }
    // An error a kernel found stays in the device control block, so the record of the newest finished gather
    // carries it: calls that enqueue work look there first and refuse once the host can know.
    void poll_status() {
        if (sticky || !ring_host) return;
        for (uint64_t g = seq; g-- > 0 && seq - g <= (uint64_t)STATS_RING;) {
            const StatsRec& rec = ring_host[g % STATS_RING];
            if (*reinterpret_cast<const volatile uint64_t*>(&rec.seq) != g) continue;   // not finished yet
            std::atomic_thread_fence(std::memory_order_acquire);
            const int32_t st = *reinterpret_cast<const volatile int32_t*>(&rec.status);
            if (st) sticky = st;
            return;
        }
    }
    uint64_t many_list_max = 1u << 20;  // merged kernels for lists up to this many raw IDs (GIDS_MANY_LIST_MAX)
    uint32_t many_meta_min = 2;         // merged calls of at least this many steps classify on the internal stream (GIDS_MANY_PIPELINE_MIN; 0: never)
    bool group_dedup = false;           // gids_cache_set_group_dedup
    char** cpu_first = nullptr;         // n_hot words, clear between merged calls (see CacheView::cpu_first)
    bool many_pool_forced = false;
    uint32_t many_chunk_forced = 0;     // GIDS_MANY_CHUNK: steps per classification launch where the sets' state is in memory
    uint64_t many_pool = 152 * 1024;    // LDS for a classifying workgroup's own list entries (GIDS_MANY_POOL, bytes; 0: none)
    int fuse = 1;               // GIDS_FUSE=0: commit, queueing and counters as a kernel each; no merged kernels
    int move_blocks = 1 << 20;  // most workgroups the row mover uses for rows that stay in HBM
    int link_blocks = 48;       // ... for rows that cross the host link (persistent)
    bool wide_index = false;    // GIDS_WIDE_INDEX=1: 64-bit set arithmetic even where 32 bits would do (for tests)
    // optional per-phase timing of each gather (events on the caller's stream)
    bool profile = false;
    hipEvent_t prof_events[STATS_RING][5] = {};   // dedup start, dedup end, metadata end, move start, move end
    bool prof_valid[STATS_RING] = {};
    int mark_phase(int ring, int phase, hipStream_t s) {
        if (!profile) return GIDS_OK;
        if (!prof_events[ring][phase]) HIP_TRY(hipEventCreate(&prof_events[ring][phase]));
        HIP_TRY(hipEventRecord(prof_events[ring][phase], s));
        return GIDS_OK;
    }
};

namespace {

template <typename IdT>
struct CacheT final : gids_cache {
    // device state
    IdT* tags = nullptr;
    int32_t* stamps = nullptr;
    uint32_t* pending = nullptr;
    uint8_t* reuse = nullptr;
    uint64_t* missmask = nullptr;
    uint64_t* bitmap = nullptr;
    uint32_t* wrank = nullptr;
    uint64_t* hotbits = nullptr;
    uint32_t* hotrank = nullptr;
    char* cache_data = nullptr;
    Ctl* ctl = nullptr;
    uint32_t* blocksum = nullptr;
    uint32_t* blockoff = nullptr;
    // per-minibatch scratch, sized for the longest raw list seen
    uint64_t cap_n = 0;
    IdT* ubuf[2] = {nullptr, nullptr};       // alternate per gather: gather t+1 is classified while the rows
    uint64_t* plan[2] = {nullptr, nullptr};  // of gather t are still moving
    BatchHdr* hdr = nullptr;                 // two entries
    // accumulator: per-line bookkeeping and the operation lists of the two groups that can exist at a time
    uint32_t* fillgrp = nullptr;
    uint32_t* hitgrp = nullptr;
    uint64_t* many_plan = nullptr;           // plan of every step of a merged call
    uint64_t many_plan_cap = 0;
    uint64_t queue_cap = 0;
    FillOp* fills[2] = {nullptr, nullptr};
    CopyOp* rcopies[2] = {nullptr, nullptr};
    CopyOp* wcopies[2] = {nullptr, nullptr};
    IdT* ustage[2] = {nullptr, nullptr};     // distinct-ID lists of the group's minibatches, until the group moves
    UniqCopies uq = {};                      // ... and where the callers want them (open group)

    AccumView accum_view() const {
        AccumView a;
        for (int k = 0; k < 2; k++) { a.fills[k] = fills[k]; a.rcopies[k] = rcopies[k]; a.wcopies[k] = wcopies[k]; }
        a.cap = queue_cap;
        return a;
    }
    // window FIFO (host bookkeeping; lists live on the device)
    std::vector<WindowSlot> slots;
    uint32_t head = 0, count = 0;
    // constant CPU buffer
    void* cpubuf_host = nullptr;
    void* cpubuf_dev = nullptr;
    uint64_t n_hot = 0;

    ~CacheT() override {
        (void)hipDeviceSynchronize();
        dev_free(tags); dev_free(stamps); dev_free(pending); dev_free(reuse); dev_free(missmask); dev_free(bitmap);
        dev_free(wrank); dev_free(hotbits); dev_free(hotrank); dev_free(cache_data); dev_free(ctl);
        dev_free(blocksum); dev_free(blockoff); dev_free(hdr);
        for (int k = 0; k < 2; k++) { dev_free(ubuf[k]); dev_free(plan[k]); }
        dev_free(fillgrp); dev_free(hitgrp); dev_free(many_plan); dev_free(cpu_first);
        for (int k = 0; k < 2; k++) { dev_free(fills[k]); dev_free(rcopies[k]); dev_free(wcopies[k]); dev_free(ustage[k]); }
        for (auto& e : ev_flush) if (e) (void)hipEventDestroy(e);
        for (auto& s : slots) if (s.ids) (void)hipFree(s.ids);
        if (cpubuf_host) (void)hipHostFree(cpubuf_host);
        if (ring_host) (void)hipHostFree(ring_host);
        for (auto& e : events) if (e) (void)hipEventDestroy(e);
        for (auto& e : ev_meta) if (e) (void)hipEventDestroy(e);
        for (auto& e : ev_hop) if (e) (void)hipEventDestroy(e);
        if (meta) (void)hipStreamDestroy(meta);
        for (auto& row : prof_events) for (auto& e : row) if (e) (void)hipEventDestroy(e);
    }

    CacheView<IdT> view() const {
        CacheView<IdT> v;
        v.n_rows = store->n_rows; v.n_sets = n_sets; v.ways = ways; v.lg_ways = lg_ways;
        v.row_bytes = store->row_bytes; v.line_bytes = line_bytes; v.words_per_set = words_per_set;
        v.use32 = (!wide_index && store->n_rows < (1ull << 32) && n_sets < (1ull << 32)) ? 1u : 0u;
        v.policy = policy; v.policy_key = policy_key; v.rows_per_line = rows_per_line;
        v.tags = tags; v.stamps = stamps; v.pending = pending; v.fillgrp = fillgrp; v.hitgrp = hitgrp; v.reuse = reuse;
        v.missmask = missmask;
        v.hotbits = n_hot ? hotbits : nullptr; v.hotrank = hotrank;
        v.cache_data = cache_data; v.store = static_cast<const char*>(store->dev);
        v.cpubuf = static_cast<const char*>(cpubuf_dev); v.ctl = ctl;
        v.cpu_first = group_dedup ? cpu_first : nullptr;
        return v;
    }

    int init() override {
        const uint64_t n_rows = store->n_rows;
        n_words = (n_rows + 63) / 64;
        const uint64_t rounds = (n_rows + n_sets - 1) / n_sets;     // IDs that share one set
        words_per_set = (uint32_t)((rounds + 63) / 64);
        int rc;
        if ((rc = dev_alloc(&tags, lines))) return rc;
        if ((rc = dev_alloc(&stamps, lines))) return rc;
        if (threshold) {
            if ((rc = dev_alloc(&pending, lines))) return rc;
            if ((rc = dev_alloc(&fillgrp, lines))) return rc;
            if ((rc = dev_alloc(&hitgrp, lines))) return rc;
        }
        if ((rc = dev_alloc(&reuse, n_rows))) return rc;
        if ((rc = dev_alloc(&missmask, n_sets * words_per_set))) return rc;
        if ((rc = dev_alloc(&bitmap, n_words))) return rc;
        if ((rc = dev_alloc(&cache_data, lines * (uint64_t)line_bytes))) return rc;
        if ((rc = dev_alloc(&ctl, 1))) return rc;
        const uint32_t nb = scan_blocks(n_words);
        if ((rc = dev_alloc(&blocksum, nb))) return rc;
        if ((rc = dev_alloc(&blockoff, nb))) return rc;
        if (sizeof(IdT) == 8) launch_fill_i64(reinterpret_cast<int64_t*>(tags), lines, -1, nullptr);
        else launch_fill_u32(reinterpret_cast<uint32_t*>(tags), lines, 0xFFFFFFFFu, nullptr);
        launch_fill_u32(reinterpret_cast<uint32_t*>(stamps), lines, 0xFFFFFFFFu, nullptr);
        if (pending) {
            launch_fill_u32(pending, lines, NO_OP, nullptr);
            launch_fill_u32(fillgrp, lines, 0xFFFFFFFFu, nullptr);
            launch_fill_u32(hitgrp, lines, 0xFFFFFFFFu, nullptr);
            for (auto& e : ev_flush) HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        }
        HIP_TRY(hipMemset(reuse, 0, n_rows));
        HIP_TRY(hipMemset(missmask, 0, n_sets * words_per_set * sizeof(uint64_t)));
        HIP_TRY(hipMemset(bitmap, 0, n_words * sizeof(uint64_t)));
        HIP_TRY(hipMemset(ctl, 0, sizeof(Ctl)));
        HIP_TRY(hipHostMalloc(reinterpret_cast<void**>(&ring_host), STATS_RING * sizeof(StatsRec), hipHostMallocMapped));
        memset(ring_host, 0xFF, STATS_RING * sizeof(StatsRec));
        HIP_TRY(hipHostGetDevicePointer(reinterpret_cast<void**>(&ring_dev), ring_host, 0));
        for (auto& e : events) HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        for (auto& e : ev_meta) HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        for (auto& e : ev_hop) HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        if ((rc = dev_alloc(&hdr, 2))) return rc;
        HIP_TRY(hipMemset(hdr, 0, 2 * sizeof(BatchHdr)));
        // Overlap costs a handful of cross-stream events per call: worth it when minibatches move megabytes.
        // Default: on for caches of 32 MiB and more; GIDS_PIPELINE=0/1 overrides.
        pipelined = lines * (uint64_t)line_bytes >= (32ull << 20);
        if (const char* env = getenv("GIDS_PIPELINE")) {
            pipelined = atoi(env) != 0;
            if (!pipelined) many_meta_min = 0;                // 0: no internal stream at all, merged calls included
        }
        if (pipelined || threshold) HIP_TRY(hipStreamCreateWithFlags(&meta, hipStreamNonBlocking));
        // one slot more than lists can be buffered: the slot a push overwrites was then read by the gather
        // before the previous one, whose rows have long moved, and not by the one still moving
        // (a cache with an accumulator can take a merged call, which pushes up to MANY_MAX lists before any of
        // them is gathered: that many slots more, so that none of them lands on a list still to be gathered)
        slots.resize(window + 2 + (threshold ? MANY_MAX : 0));
        if (const char* env = getenv("GIDS_WIDE_INDEX")) wide_index = atoi(env) != 0;
        if (const char* env = getenv("GIDS_FUSE")) fuse = atoi(env) & 1;
        if (const char* env = getenv("GIDS_MANY_LIST_MAX")) many_list_max = (uint64_t)std::max(0ll, atoll(env));
        if (const char* env = getenv("GIDS_MANY_POOL")) {     // (as given, whether the lists fit it or not)
            many_pool = (uint64_t)std::max(0ll, atoll(env));
            many_pool_forced = true;
        }
        if (const char* env = getenv("GIDS_MANY_PIPELINE_MIN")) many_meta_min = (uint32_t)std::max(0, atoi(env));
        if (const char* env = getenv("GIDS_MANY_CHUNK")) many_chunk_forced = (uint32_t)std::max(0, atoi(env));
        if (const char* env = getenv("GIDS_MOVE_BLOCKS")) {
            const int b = atoi(env);
            if (b >= 1 && b <= (1 << 20)) move_blocks = b;
        }
        if (const char* env = getenv("GIDS_LINK_BLOCKS")) {
            const int b = atoi(env);
            if (b >= 1 && b <= 65536) link_blocks = b;
        }
        HIP_TRY(hipDeviceSynchronize());
        return GIDS_OK;
    }

    // scratch for lists of up to n raw IDs; queues for threshold + n rows
    int ensure_scratch(uint64_t n) {
        if (n < 1) n = 1;
        if (n > cap_n) {
            HIP_TRY(hipDeviceSynchronize());
            const uint64_t want = std::max<uint64_t>(n, cap_n + cap_n / 2);
            cap_n = 0;
            for (int k = 0; k < 2; k++) {
                dev_free(ubuf[k]); dev_free(plan[k]);
                int rc;
                if ((rc = dev_alloc(&ubuf[k], want))) return rc;
                if ((rc = dev_alloc(&plan[k], want))) return rc;
            }
            cap_n = want;
        }
        return GIDS_OK;
    }

    // room for `rows` operations in each list of both groups; what is queued survives a move
    // the table behind gids_cache_set_group_dedup, once it is asked for and a CPU buffer exists
    int ensure_cpu_first() {
        if (!group_dedup || !n_hot || cpu_first) return GIDS_OK;
        int rc = dev_alloc(&cpu_first, n_hot);
        if (rc) return rc;
        HIP_TRY(hipMemset(cpu_first, 0, n_hot * sizeof(char*)));
        return GIDS_OK;
    }

    int ensure_queue(uint64_t rows) {
        if (rows <= queue_cap) return GIDS_OK;
        HIP_TRY(hipDeviceSynchronize());
        const uint64_t want = std::max<uint64_t>(rows, queue_cap + queue_cap / 2);
        for (int k = 0; k < 2; k++) {
            FillOp* nf = nullptr;
            CopyOp *nr = nullptr, *nw = nullptr;
            IdT* nu = nullptr;
            int rc;
            if ((rc = dev_alloc(&nf, want)) || (rc = dev_alloc(&nr, want)) || (rc = dev_alloc(&nw, want)) ||
                (rc = dev_alloc(&nu, want))) {
                dev_free(nf); dev_free(nr); dev_free(nw); dev_free(nu);
                return rc;
            }
            if (queue_cap) {
                HIP_TRY(hipMemcpy(nf, fills[k], queue_cap * sizeof(FillOp), hipMemcpyDeviceToDevice));
                HIP_TRY(hipMemcpy(nr, rcopies[k], queue_cap * sizeof(CopyOp), hipMemcpyDeviceToDevice));
                HIP_TRY(hipMemcpy(nw, wcopies[k], queue_cap * sizeof(CopyOp), hipMemcpyDeviceToDevice));
                HIP_TRY(hipMemcpy(nu, ustage[k], queue_cap * sizeof(IdT), hipMemcpyDeviceToDevice));
            }
            dev_free(fills[k]); dev_free(rcopies[k]); dev_free(wcopies[k]); dev_free(ustage[k]);
            fills[k] = nf; rcopies[k] = nr; wcopies[k] = nw; ustage[k] = nu;
        }
        queue_cap = want;
        return GIDS_OK;
    }

    int ensure_slot(WindowSlot& s, uint64_t n) {
        if (n < 1) n = 1;
        if (n <= s.cap) return GIDS_OK;
        HIP_TRY(hipDeviceSynchronize());
        if (s.ids) (void)hipFree(s.ids);
        s.ids = nullptr; s.cap = 0;
        HIP_TRY(hipMalloc(&s.ids, n * sizeof(IdT)));
        s.cap = n;
        return GIDS_OK;
    }

    int reserve(uint64_t n) override {
        int rc = ensure_scratch(n);
        if (rc) return rc;
        // a group closes once it holds the threshold's node accesses: at most one list beyond it (the adaptive
        // mode raises the threshold by up to its bound)
        if (threshold) {
            const uint64_t t_max = accum_mode == GIDS_ACCUM_ADAPTIVE ? threshold * ACCUM_MAX_RAISE : threshold;
            if ((rc = ensure_queue(std::min<uint64_t>(t_max + n, (uint64_t)ACCUM_MAX_MERGE * std::max<uint64_t>(n, 1))))) return rc;
        }
        for (auto& s : slots) {
            // only lists that are not in use may move
            bool live = false;
            for (uint32_t k = 0; k < count; k++) live |= (&s == &slots[(head + k) % slots.size()]);
            if (!live && (rc = ensure_slot(s, n))) return rc;
        }
        return GIDS_OK;
    }

    int pin(const void* ids_host, uint64_t n) override {
        if (n_hot || seq || count) return fail(GIDS_E_INVAL, "gids_cpu_buffer_pin: call once, before any push or gather");
        if (n == 0) return GIDS_OK;
        if (!ids_host) return fail(GIDS_E_INVAL, "gids_cpu_buffer_pin: ids_host is NULL");
        const IdT* ids = static_cast<const IdT*>(ids_host);
        std::vector<uint64_t> sorted(n);
        for (uint64_t i = 0; i < n; i++) {
            if (ids[i] < 0 || (uint64_t)ids[i] >= store->n_rows) return fail(GIDS_E_RANGE, "gids_cpu_buffer_pin: ID %lld out of range", (long long)ids[i]);
            sorted[i] = (uint64_t)ids[i];
        }
        std::sort(sorted.begin(), sorted.end());
        for (uint64_t i = 1; i < n; i++)
            if (sorted[i] == sorted[i - 1]) return fail(GIDS_E_INVAL, "gids_cpu_buffer_pin: ID %llu listed twice", (unsigned long long)sorted[i]);
        const uint64_t rb = store->row_bytes;
        const int rc_alloc = pin_alloc(n * rb);
        if (rc_alloc) { pin_release(); return rc_alloc; }
        // rows in ascending ID order: slot = rank of the ID among the pinned ones
        {
            const unsigned hw = std::max(1u, std::min(16u, std::thread::hardware_concurrency()));
            const unsigned nt = (unsigned)std::min<uint64_t>(hw, std::max<uint64_t>(1, n * rb >> 24));
            std::vector<std::thread> pool;
            const char* src = static_cast<const char*>(store->host);
            char* dst = static_cast<char*>(cpubuf_host);
            for (unsigned t = 0; t < nt; t++)
                pool.emplace_back([&, t]() {
                    for (uint64_t i = n * t / nt; i < n * (t + 1) / nt; i++) memcpy(dst + i * rb, src + sorted[i] * rb, rb);
                });
            for (auto& th : pool) th.join();
        }
        std::vector<uint64_t> bits(n_words, 0);
        std::vector<uint32_t> rank(n_words, 0);
        for (uint64_t v : sorted) bits[v >> 6] |= 1ull << (v & 63);
        uint32_t run = 0;
        for (uint64_t w = 0; w < n_words; w++) { rank[w] = run; run += (uint32_t)__builtin_popcountll(bits[w]); }
        const int rc = pin_upload(bits, rank);
        if (rc) { pin_release(); return rc; }
        n_hot = n;
        return GIDS_OK;
    }

    int pin_alloc(uint64_t bytes) {
        HIP_TRY(hipHostMalloc(&cpubuf_host, bytes, hipHostMallocMapped));
        HIP_TRY(hipHostGetDevicePointer(&cpubuf_dev, cpubuf_host, 0));
        return GIDS_OK;
    }
    int pin_upload(const std::vector<uint64_t>& bits, const std::vector<uint32_t>& rank) {
        int rc;
        if ((rc = dev_alloc(&hotbits, n_words))) return rc;
        if ((rc = dev_alloc(&hotrank, n_words))) return rc;
        HIP_TRY(hipMemcpy(hotbits, bits.data(), n_words * sizeof(uint64_t), hipMemcpyHostToDevice));
        HIP_TRY(hipMemcpy(hotrank, rank.data(), n_words * sizeof(uint32_t), hipMemcpyHostToDevice));
        return GIDS_OK;
    }
    // a pin that failed half-way leaves the cache as it was, without a CPU buffer
    void pin_release() {
        if (cpubuf_host) (void)hipHostFree(cpubuf_host);
        cpubuf_host = cpubuf_dev = nullptr;
        dev_free(hotbits); dev_free(hotrank);
    }

    // ascending distinct IDs of ids[0..n) -> dst; count -> *n_out (device)
    void dedup(const IdT* ids, uint64_t n, IdT* dst, uint32_t* n_out, uint8_t* reuse_inc, bool keep_bitmap,
               hipStream_t s, const uint32_t* n_dev = nullptr) {
        launch_mark<IdT>(ids, n, n_dev, store->n_rows, bitmap, ctl, s);
        // a bitmap that one block scans needs no separate count: that block's total is the distinct count
        const bool solo = scan_blocks(n_words) == 1;
        if (!solo) launch_count(bitmap, n_words, blocksum, blockoff, ctl, n_out, s);
        launch_emit<IdT>(bitmap, n_words, store->n_rows, blockoff, dst, reuse_inc, keep_bitmap ? wrank : nullptr,
                         !keep_bitmap, ctl, solo ? n_out : nullptr, s);
    }

    int push(const void* ids, uint64_t n, const uint32_t* n_dev, hipStream_t s) override {
        if (count == window + 1) return fail(GIDS_E_FULL, "gids_window_push: %u lists already buffered", count);
        if (n && !ids) return fail(GIDS_E_INVAL, "gids_window_push: ids_dev is NULL");
        const uint32_t slot = (head + count) % slots.size();
        WindowSlot& sl = slots[slot];
        int rc = ensure_slot(sl, n);
        if (rc) return rc;
        sl.n_raw = n;
        // From here on kernels of this push may already be queued when a later HIP call fails: the device
        // state would then be ahead of the host's bookkeeping, so such a failure closes the cache.
        if ((rc = push_enqueue(static_cast<const IdT*>(ids), n, n_dev, slot, s))) sticky = rc;
        return rc;
    }

    int push_enqueue(const IdT* ids, uint64_t n, const uint32_t* n_dev, uint32_t slot, hipStream_t s) {
        WindowSlot& sl = slots[slot];
        int rc;
        if ((rc = follow(s))) return rc;
        hipStream_t m = s;
        if (pipelined) {
            m = meta;
            // the list this slot held may still be read by its gather's row mover
            // (not with the accumulator: there the list is last read by the queue kernel, on this same stream)
            if (sl.last_reader >= 0 && !threshold) HIP_TRY(hipStreamWaitEvent(meta, events[sl.last_reader % STATS_RING], 0));
            if ((rc = edge(s, meta))) return rc;              // the caller's IDs are ready in its stream's order
        }
        dedup(ids, n, static_cast<IdT*>(sl.ids), &ctl->win_n[slot], reuse, false, m, n_dev);
        if (pipelined && (rc = edge(meta, s))) return rc;     // the caller may reuse its ID buffer in stream order
        HIP_TRY(hipGetLastError());                           // a kernel launch that was refused
        sl.last_reader = -1;
        count++;
        return GIDS_OK;
    }

    // the per-gather buffers of one parity: the library's own, or their places in the static workspace
    struct GatherBufs {
        IdT* ub;
        uint64_t* pl;
        BatchHdr* hd;
    };

    int gather(const void* ids_v, uint64_t n, void* out, uint64_t out_cap, void* unique, void* inverse,
               bool no_alloc, hipStream_t s) override {
        const IdT* ids = static_cast<const IdT*>(ids_v);
        if (!out && out_cap) return fail(GIDS_E_INVAL, "gids_gather: out_dev is NULL");
        if (inverse && !ids) return fail(GIDS_E_INVAL, "gids_gather: inverse_dev needs ids_dev");
        if (window && count == 0) return fail(GIDS_E_ORDER, "gids_gather: no minibatch is buffered in the window");
        // With window_depth 0 a list may still have been pushed ahead (it pins nothing: its counters are back
        // at zero before any victim is chosen); then it is the minibatch, exactly as with a window.
        const bool head_list = window != 0 || count != 0;
        if (!head_list && !ids && n) return fail(GIDS_E_INVAL, "gids_gather: ids_dev is NULL and no list was pushed to take it from");
        if (!ids) n = 0;
        const uint64_t longest = head_list ? std::max(n, slots[head].n_raw) : n;
        const int par = (int)(seq & 1);
        GatherBufs b;
        int rc;
        if (no_alloc) {
            if (threshold) return fail(GIDS_E_INVAL, "gids_gather_static: not on a cache with accum_threshold > 0 (its operation lists grow on demand)");
            if (longest > STATIC_MAX_IDS) return fail(GIDS_E_INVAL, "gids_gather_static: a list of %llu IDs exceeds the static workspace (GIDS_STATIC_MAX_IDS = %llu)", (unsigned long long)longest, (unsigned long long)STATIC_MAX_IDS);
            unsigned char* ws = static_cast<unsigned char*>(static_ws);
            b.hd = reinterpret_cast<BatchHdr*>(ws) + par;
            b.pl = reinterpret_cast<uint64_t*>(ws + STATIC_HDR_BYTES) + (uint64_t)par * STATIC_MAX_IDS;
            b.ub = reinterpret_cast<IdT*>(ws + STATIC_HDR_BYTES + (2 + (uint64_t)par) * STATIC_MAX_IDS * sizeof(uint64_t));
        } else {
            if ((rc = ensure_scratch(longest))) return rc;
            if (inverse && !wrank && (rc = dev_alloc(&wrank, n_words))) return rc;
            b.hd = hdr + par; b.pl = plan[par]; b.ub = ubuf[par];
        }
        // (as in push: a HIP failure once kernels may be queued closes the cache)
        const bool was_profiling = profile;
        if (no_alloc) profile = false;                        // phase events are created on first use
        rc = gather_enqueue(ids, n, head_list, b, out, out_cap, unique, inverse, s);
        profile = was_profiling;
        if (rc) sticky = rc;
        return rc;
    }

    // Node-access threshold of the open group.  Fixed mode: accum_threshold.  Adaptive mode (Section 3.2, last
    // paragraph): accum_threshold is the number of store accesses wanted in flight, and since part of the node
    // accesses is redirected to the GPU cache and the CPU buffer, the node-access threshold is that number times
    // (node accesses / store accesses), measured over every gather at least ACCUM_LAG calls back (a fixed lag,
    // so the groups do not depend on how far the device has got; the call waits for those counters if need be).
    int accum_limit(uint64_t* limit) {
        *limit = threshold;
        if (accum_mode != GIDS_ACCUM_ADAPTIVE) return GIDS_OK;
        while (adapt_next + ACCUM_LAG < seq) {
            const uint64_t g = adapt_next;
            const int r = (int)(g % STATS_RING);
            if (pipelined) HIP_TRY(hipEventSynchronize(ev_meta[ev_of[r]]));
            HIP_TRY(hipEventSynchronize(events[ev_of[r]]));
            const StatsRec& rec = ring_host[r];
            if (*reinterpret_cast<const volatile uint64_t*>(&rec.seq) != g) return fail(GIDS_E_HIP, "the counters of gather %llu are missing", (unsigned long long)g);
            adapt_nodes += raw_of[r];
            adapt_store += *reinterpret_cast<const volatile uint64_t*>(&rec.n_miss);
            adapt_next++;
        }
        if (adapt_nodes == 0) return GIDS_OK;
        const uint64_t top = threshold * ACCUM_MAX_RAISE;
        if (adapt_store == 0) { *limit = top; return GIDS_OK; }
        const unsigned __int128 want = ((unsigned __int128)threshold * adapt_nodes + adapt_store - 1) / adapt_store;
        *limit = want > top ? top : std::max<uint64_t>(threshold, (uint64_t)want);
        return GIDS_OK;
    }

    int gather_enqueue(const IdT* ids, uint64_t n, bool head_list, const GatherBufs& b, void* out, uint64_t out_cap,
                       void* unique, void* inverse, hipStream_t s) {
        int rc;
        const int r = (int)(seq % STATS_RING);
        const uint64_t n_raw = head_list ? slots[head].n_raw : n;
        const uint64_t n_upper = std::min<uint64_t>(n_raw, store->n_rows);
        // the accumulator's decision, taken here on what the host knows: does this gather close its group?
        bool opens = false, closes = false;
        uint64_t limit = 0;
        if (threshold) {
            if ((rc = accum_limit(&limit))) return rc;
            opens = open_batches == 0;
            if ((rc = ensure_queue(open_upper + n_upper))) return rc;
            if ((rc = ensure_cpu_first())) return rc;
            closes = open_nodes + n_raw >= limit || open_batches + 1 >= ACCUM_MAX_MERGE;
            if (group_override) closes = group_override == 2; // a merged call decides for itself
        }
        if ((rc = follow(s))) return rc;
        hipStream_t m = s;
        if (pipelined) {
            m = meta;
            // plan / ID scratch / header of this parity were last read by the row mover of gather seq - 2
            // (with the accumulator by this stream's own queue kernel)
            if (seq >= 2 && !threshold) HIP_TRY(hipStreamWaitEvent(meta, events[(seq - 2) % STATS_RING], 0));
            if (ids && (rc = edge(s, meta))) return rc;       // the caller's IDs are ready in its stream's order
        }
        // the lists this group will fill were last read by the group mover two groups back
        if (opens && flush_recorded[group & 1]) HIP_TRY(hipStreamWaitEvent(m, ev_flush[group & 1], 0));
        prof_valid[r] = false;
        if ((rc = mark_phase(r, 0, m))) return rc;

        const IdT* U;
        const uint32_t* n_u;
        if (ids || !head_list) {                              // (an empty list without a window still sets the count)
            dedup(ids, n, b.ub, &ctl->n_unique, nullptr, inverse != nullptr, m);
            if (head_list)
                launch_verify<IdT>(b.ub, static_cast<const IdT*>(slots[head].ids), &ctl->win_n[head], ctl,
                                   std::min(n, slots[head].n_raw), m);
            if (inverse) {
                launch_inverse<IdT>(ids, n, bitmap, wrank, static_cast<uint32_t*>(inverse), ctl, m);
                launch_clear<IdT>(bitmap, b.ub, &ctl->n_unique, n, m);
            }
        }
        if (head_list) {                                      // the buffered head list is the minibatch
            U = static_cast<const IdT*>(slots[head].ids);
            n_u = &ctl->win_n[head];
        } else {
            U = b.ub;
            n_u = &ctl->n_unique;
        }
        const CacheView<IdT> c = view();
        if ((rc = mark_phase(r, 1, m))) return rc;
        const int accum_flags = threshold ? 4 | (closes ? 1 : 0) | (opens ? 2 : 0) | (int)((group & 1) << 3) | (int)(open_batches << 8) : 0;
        // with the accumulator the distinct-ID list is staged in the group's buffer (this stream may run ahead of
        // the caller's) and copied to the caller's buffer when the group moves
        IdT* unique_to = static_cast<IdT*>(unique);
        if (threshold) {
            uq.dst[open_batches] = unique;
            uq.src_entry[open_batches] = open_upper;
            uq.n = open_batches + 1;
            unique_to = unique ? ustage[group & 1] + open_upper : nullptr;
        }
        launch_probe<IdT>(c, U, n_u, n_upper, out_cap, head_list, b.pl, m);
        launch_victim<IdT>(c, U, n_u, n_upper, b.pl, m);
        // commit, queueing and counters: one launch, or (GIDS_FUSE without bit 0) a kernel each
        const bool settle = (fuse & 1) != 0;
        if (settle) {
            launch_settle<IdT>(c, accum_view(), group, accum_flags, U, n_u, n_upper, b.pl, b.hd, static_cast<char*>(out),
                               unique_to, ring_dev + r, seq, m);
        } else {
            launch_commit<IdT>(c, U, n_u, n_upper, b.pl, b.hd, m);
        }
        if (threshold == 0) {
            if (!settle) launch_finalize(ctl, ring_dev + r, seq, n_u, 0, m);
            if ((rc = mark_phase(r, 2, m))) return rc;
            if (pipelined) {
                HIP_TRY(hipEventRecord(ev_meta[r], meta));
                HIP_TRY(hipStreamWaitEvent(s, ev_meta[r], 0));
            }
            if ((rc = mark_phase(r, 3, s))) return rc;
            launch_move<IdT>(c, U, b.hd, n_upper, b.pl, static_cast<char*>(out), static_cast<IdT*>(unique),
                             move_blocks, link_blocks, s);
            if ((rc = mark_phase(r, 4, s))) return rc;
        } else {
            // nothing moves yet: the minibatch's rows join the open group's lists (on the metadata stream, so
            // that the next minibatch is classified while an earlier group is still moving)
            if (!settle) {
                launch_queue<IdT>(c, accum_view(), group, U, b.hd, n_upper, b.pl, static_cast<char*>(out), unique_to, m);
                launch_finalize(ctl, ring_dev + r, seq, n_u, accum_flags, m);
            }
            // (the words that remember the group's first fill of a CPU-buffer row are clear between groups)
            if (closes && group_dedup && cpu_first) launch_fill_i64(reinterpret_cast<int64_t*>(cpu_first), n_hot, 0, m);
            if ((rc = mark_phase(r, 2, m))) return rc;
            raw_of[r] = (uint32_t)n_raw;
            open_nodes += n_raw;
            open_upper += n_upper;
            open_batches++;
            if (pipelined) HIP_TRY(hipEventRecord(ev_meta[r], meta));
            if ((rc = mark_phase(r, 3, s))) return rc;
            if (closes && (rc = close_group(s, pipelined ? ev_meta[r] : nullptr))) return rc;
            if ((rc = mark_phase(r, 4, s))) return rc;
        }
        prof_valid[r] = profile;
        ev_of[r] = r;
        HIP_TRY(hipGetLastError());                           // a kernel launch that was refused
        HIP_TRY(hipEventRecord(events[r], s));
        if (head_list) {
            slots[head].last_reader = (int64_t)seq;
            head = (head + 1) % slots.size();
            count--;
        }
        seq++;
        return GIDS_OK;
    }

    // the rows of the open group move, in two launches on the caller's stream
    int close_group(hipStream_t s, hipEvent_t after) {
        const uint32_t par = group & 1;
        if (after) HIP_TRY(hipStreamWaitEvent(s, after, 0));
        launch_group_move<IdT>(view(), accum_view(), par, open_upper, move_blocks, link_blocks, uq, ustage[par], s);
        uq.n = 0;
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipEventRecord(ev_flush[par], s));
        flush_recorded[par] = true;
        group++;
        open_nodes = open_upper = 0;
        open_batches = 0;
        return GIDS_OK;
    }

    int flush(hipStream_t s) override {
        if (!threshold || open_batches == 0) return GIDS_OK;
        int rc = flush_enqueue(s);
        if (rc) sticky = rc;
        return rc;
    }

    int flush_enqueue(hipStream_t s) {
        int rc = follow(s);
        if (rc) return rc;
        if (group_dedup && cpu_first) launch_fill_i64(reinterpret_cast<int64_t*>(cpu_first), n_hot, 0, pipelined ? meta : s);
        hipEvent_t after = nullptr;
        if (pipelined) {                                      // everything the open group's gathers queued
            after = ev_hop[hop++ % 16];
            HIP_TRY(hipEventRecord(after, meta));
        }
        return close_group(s, after);
    }

    // k steps, each "push one list (optional), gather the window's head", as one accumulator group.
    int gather_many(uint32_t k, const void* const* push_ids, const uint64_t* push_n, void* const* outs,
                    const uint64_t* caps, void* const* uniques, hipStream_t ps, hipStream_t s) override {
        if (!threshold) return fail(GIDS_E_INVAL, "gids_gather_many: the cache was created without an accumulator (accum_threshold == 0)");
        if (k < 1 || k > (uint32_t)MANY_MAX) return fail(GIDS_E_INVAL, "gids_gather_many: k must be in [1, %d]", MANY_MAX);
        if (!outs || !caps) return fail(GIDS_E_INVAL, "gids_gather_many: out_dev / out_capacity_rows is NULL");
        // the window protocol over the whole call, before anything is enqueued
        uint32_t cnt = count;
        uint64_t total_upper = 0;
        for (uint32_t i = 0; i < k; i++) {
            const bool pushes = push_ids && push_ids[i];
            if (pushes) {
                if (push_n[i] > 0xFFFFFFF0ull) return fail(GIDS_E_INVAL, "gids_gather_many: list %u too long", i);
                if (cnt == window + 1) return fail(GIDS_E_FULL, "gids_gather_many: step %u pushes into a full window", i);
                cnt++;
            }
            if (cnt == 0) return fail(GIDS_E_ORDER, "gids_gather_many: step %u has no buffered minibatch to gather", i);
            cnt--;
            if (!outs[i] && caps[i]) return fail(GIDS_E_INVAL, "gids_gather_many: out_dev[%u] is NULL", i);
        }
        // The merged kernels want a workgroup's share of every list in its LDS (many_fits): a workgroup whose
        // share does not fit reads all the lists from memory in every phase of every step, which for lists of
        // tens of thousands of IDs costs more than the per-step kernels as one group.
        uint64_t longest_raw = 0;
        {
            uint32_t h = head, c2 = count;
            std::vector<uint64_t> len(slots.size());
            for (size_t q = 0; q < slots.size(); q++) len[q] = slots[q].n_raw;
            for (uint32_t i = 0; i < k; i++) {
                if (push_ids && push_ids[i]) {
                    len[(h + c2) % slots.size()] = push_n[i];
                    longest_raw = std::max(longest_raw, push_n[i]);
                    c2++;
                }
                longest_raw = std::max(longest_raw, len[h]);
                h = (h + 1) % slots.size();
                c2--;
            }
        }
        // the window slots the steps will read, as many_enqueue will assign them
        std::vector<int> pushed_at(k, -1), head_at(k, 0);
        {
            uint32_t h = head, c2 = count;
            for (uint32_t i = 0; i < k; i++) {
                if (push_ids && push_ids[i]) {
                    pushed_at[i] = (int)((h + c2) % slots.size());
                    c2++;
                }
                head_at[i] = (int)h;
                h = (h + 1) % slots.size();
                c2--;
            }
        }
        auto lists_between = [&](uint32_t a, uint32_t b) {    // distinct lists the steps [a, b) read
            std::vector<char> seen(slots.size(), 0);
            uint32_t n = 0;
            for (uint32_t i = a; i < b; i++) {
                if (pushed_at[i] >= 0 && !seen[pushed_at[i]]) { seen[pushed_at[i]] = 1; n++; }
                if (!seen[head_at[i]]) { seen[head_at[i]] = 1; n++; }
            }
            return n;
        };
        // What the classification is sized for: the longest list's distinct IDs.  The host knows raw lengths only;
        // the finished gathers tell how many distinct IDs a raw list of this stream tends to hold.
        update_distinct_ratio();
        const uint64_t longest_est = std::max<uint64_t>(1, std::min<uint64_t>(store->n_rows,
            (uint64_t)std::ceil((double)longest_raw * std::min(1.0, distinct_ratio * 1.25))));
        // steps per launch of the classification: all of them where their lists fit a workgroup's LDS together;
        // fewer where the sets' state stays in device memory anyway (a launch then leaves nothing behind in LDS
        // that the next would miss); 0: the per-step kernels
        uint32_t chunk = 0;
        if (store->n_rows < (1ull << 32) && n_sets < (1ull << 32) && ways <= many_max_ways() && rows_per_line == 1 &&
            (fuse & 1) && longest_raw <= many_list_max) {
            bool in_lds = false;
            auto fits = [&](uint32_t n_lists) {
                return many_fits(store->n_rows, n_sets, ways, words_per_set, sizeof(IdT), n_lists, longest_est, many_pool,
                                 group_dedup, &in_lds);
            };
            const bool all_fit = fits(lists_between(0, k));
            if (many_chunk_forced && many_chunk_forced < k && !in_lds) {
                chunk = many_chunk_forced;
            } else if (many_pool_forced || all_fit) {
                chunk = k;
            } else if (!in_lds) {
                for (uint32_t c : {16u, 8u, 4u}) {
                    if (c >= k) continue;
                    uint32_t most = 0;
                    for (uint32_t a = 0; a < k; a += c) most = std::max(most, lists_between(a, std::min(k, a + c)));
                    if (fits(most)) { chunk = c; break; }
                }
            }
        }
        const bool fast = chunk != 0;
        int rc;
        if (!fast) {
            // large tables, high associativity: the same steps through the per-step kernels, still one group
            many_slow_calls++;
            if (open_batches && (rc = flush(s))) return rc;
            for (uint32_t i = 0; i < k; i++) {
                if (push_ids && push_ids[i] && (rc = push(push_ids[i], push_n[i], nullptr, ps))) return rc;
                group_override = i + 1 < k ? 1 : 2;           // no group closes inside the call, its last step closes it
                rc = gather(nullptr, 0, outs[i], caps[i], uniques ? uniques[i] : nullptr, nullptr, false, s);
                group_override = 0;
                if (rc) return rc;
            }
            return GIDS_OK;
        }
        many_fast_calls++;
        if ((rc = ensure_cpu_first())) return rc;
        // room: window slots of the pushed lists, the plans of all steps, the group's lists
        if (open_batches && (rc = flush(s))) return rc;
        {
            uint32_t h = head, c2 = count;
            for (uint32_t i = 0; i < k; i++) {
                if (push_ids && push_ids[i]) {
                    WindowSlot& sl = slots[(h + c2) % slots.size()];
                    if ((rc = ensure_slot(sl, push_n[i]))) return rc;
                    sl.n_raw = push_n[i];
                    c2++;
                }
                const uint64_t up = std::min<uint64_t>(slots[h].n_raw, store->n_rows);
                total_upper += up;
                h = (h + 1) % slots.size();
                c2--;
            }
        }
        if (total_upper > many_plan_cap) {
            HIP_TRY(hipDeviceSynchronize());
            dev_free(many_plan);
            many_plan_cap = 0;
            if ((rc = dev_alloc(&many_plan, total_upper + total_upper / 2))) return rc;
            many_plan_cap = total_upper + total_upper / 2;
        }
        if ((rc = ensure_queue(total_upper))) return rc;
        if ((rc = many_enqueue(k, chunk, push_ids, push_n, outs, caps, uniques, total_upper, std::max<uint64_t>(longest_est, 1), ps, s))) sticky = rc;
        return rc;
    }

    int many_enqueue(uint32_t k, uint32_t chunk, const void* const* push_ids, const uint64_t* push_n, void* const* outs,
                     const uint64_t* caps, void* const* uniques, uint64_t total_upper, uint64_t longest, hipStream_t ps,
                     hipStream_t s) {
        int rc;
        const bool any_push = push_ids != nullptr;
        // A call of several steps classifies on the internal stream also where the cache is too small for single
        // gathers to do so: one pair of cross-stream waits per call, and the classification of this call runs
        // beside the row movement of the call before (Tiny, us per minibatch with / without: 39 / 49 for calls of
        // two steps, 22 / 30 of four, 14 / 20 of eight, 10 / 15 of sixteen).
        const bool on_meta = pipelined || (many_meta_min && k >= many_meta_min);
        hipStream_t m = s;
        if (on_meta) {
            m = meta;
            if (!pipelined) {                                 // after whatever the one-stream calls before have queued
                if (have_last && one_stream_work && (rc = edge(last_stream, meta))) return rc;
                one_stream_work = false;
                last_stream = s;                              // (this call's row movement, behind its classification)
                have_last = true;
            }
            if (any_push && (rc = edge(ps, meta))) return rc; // the caller's ID lists are ready in the push stream's order
        } else {
            if (any_push && (rc = follow(ps))) return rc;
            if ((rc = follow(s))) return rc;
        }
        if (flush_recorded[group & 1]) HIP_TRY(hipStreamWaitEvent(m, ev_flush[group & 1], 0));
        // the steps' bookkeeping (window slots, outputs, staging of the distinct-ID lists) and the pushed lists
        ManyPushes<IdT> mp;
        struct Step { int pushed_slot; uint32_t head_slot; uint64_t plan_offset; };
        std::vector<Step> steps(k);
        uint32_t n_push = 0;
        uint64_t off = 0;
        for (uint32_t i = 0; i < k; i++) {
            steps[i].pushed_slot = -1;
            if (push_ids && push_ids[i]) {
                const uint32_t slot = (head + count) % slots.size();
                WindowSlot& sl = slots[slot];
                mp.ids[n_push] = static_cast<const IdT*>(push_ids[i]);
                mp.n[n_push] = push_n[i];
                mp.dst[n_push] = static_cast<IdT*>(sl.ids);
                mp.slot[n_push] = slot;
                n_push++;
                steps[i].pushed_slot = (int)slot;
                sl.last_reader = -1;
                count++;
            }
            const uint64_t n_raw = slots[head].n_raw;
            steps[i].head_slot = head;
            steps[i].plan_offset = off;
            off += std::min<uint64_t>(n_raw, store->n_rows);
            uq.dst[i] = uniques ? uniques[i] : nullptr;       // staged, and copied out when the group moves
            uq.src_entry[i] = steps[i].plan_offset;
            const int r = (int)((seq + i) % STATS_RING);
            raw_of[r] = (uint32_t)n_raw;
            prof_valid[r] = false;
            slots[head].last_reader = (int64_t)(seq + i);
            head = (head + 1) % slots.size();
            count--;
        }
        if (store->n_rows <= many_max_rows()) {
            launch_dedup_small<IdT>(mp, n_push, store->n_rows, ctl, m);
        } else {
            // a table whose bitmap does not fit a workgroup's LDS: the pushed lists go through the bitmap in
            // device memory one after the other; their future-reuse counters are raised by the classification,
            // step by step, as for the lists above
            for (uint32_t q = 0; q < n_push; q++)
                dedup(mp.ids[q], mp.n[q], mp.dst[q], &ctl->win_n[mp.slot[q]], nullptr, false, m);
        }
        // the caller's ID buffers are read by that kernel alone: the push stream goes on as soon as it is through
        // (were it held until the classification ends, the next call's lists would be ready that much later)
        if (on_meta && n_push && (rc = edge(meta, ps))) return rc;
        // the classification: one launch for the steps [a, b) at a time (all of them where their lists fit a
        // workgroup's LDS together), the group staying open in between
        for (uint32_t a = 0; a < k; a += chunk) {
            const uint32_t b = std::min(k, a + chunk);
            ManySteps<IdT> ms;
            ms.k = b - a;
            ms.seq0 = seq + a;
            ms.step0 = a;
            ms.closes_group = b == k ? 1u : 0u;
            ms.group_dedup = group_dedup ? 1u : 0u;
            ms.n_lists = 0;
            std::vector<int> list_of_slot(slots.size(), -1);
            auto list_of = [&](uint32_t slot, bool is_head) {
                int& l = list_of_slot[slot];
                if (l < 0) {
                    l = (int)ms.n_lists++;
                    ms.list[l] = static_cast<const IdT*>(slots[slot].ids);
                    ms.list_slot[l] = (uint16_t)slot;
                    ms.list_is_head[l] = 0;
                }
                if (is_head) ms.list_is_head[l] = 1;
                return (uint8_t)l;
            };
            for (uint32_t i = a; i < b; i++) {
                const uint32_t x = i - a;
                ms.pushed[x] = nullptr;
                ms.pushed_slot[x] = 0;
                ms.pushed_list[x] = MANY_NO_LIST;
                if (steps[i].pushed_slot >= 0) {
                    const uint32_t slot = (uint32_t)steps[i].pushed_slot;
                    ms.pushed[x] = static_cast<const IdT*>(slots[slot].ids);
                    ms.pushed_slot[x] = slot;
                    ms.pushed_list[x] = list_of(slot, false);
                }
                ms.head_list[x] = list_of(steps[i].head_slot, true);
                ms.head[x] = static_cast<const IdT*>(slots[steps[i].head_slot].ids);
                ms.head_slot[x] = steps[i].head_slot;
                ms.out_capacity[x] = caps[i];
                ms.plan_offset[x] = steps[i].plan_offset;
                ms.out[x] = static_cast<char*>(outs[i]);
                ms.unique_out[x] = uq.dst[i] ? ustage[group & 1] + steps[i].plan_offset : nullptr;
            }
            launch_classify_many<IdT>(view(), accum_view(), group, ms, longest, many_pool, many_plan, ring_dev, STATS_RING, m);
        }
        // (a call in several launches: the words that remember the first fill of a CPU-buffer row are cleared here)
        if (chunk < k && group_dedup && cpu_first)
            launch_fill_i64(reinterpret_cast<int64_t*>(cpu_first), n_hot, 0, m);
        HIP_TRY(hipGetLastError());
        const int r_last = (int)((seq + k - 1) % STATS_RING);
        for (uint32_t i = 0; i < k; i++) ev_of[(seq + i) % STATS_RING] = r_last;
        if (on_meta) HIP_TRY(hipEventRecord(ev_meta[r_last], meta));
        open_upper = total_upper;
        open_batches = k;
        uq.n = k;
        seq += k;
        if ((rc = close_group(s, on_meta ? ev_meta[r_last] : nullptr))) return rc;
        HIP_TRY(hipEventRecord(events[r_last], s));
        return GIDS_OK;
    }

    uint32_t window_count() const override { return count; }

    int snapshot(int64_t* tags_host, int64_t* stamps_host) override {
        HIP_TRY(hipDeviceSynchronize());
        if (tags_host) {
            std::vector<IdT> t(lines);
            HIP_TRY(hipMemcpy(t.data(), tags, lines * sizeof(IdT), hipMemcpyDeviceToHost));
            for (uint64_t i = 0; i < lines; i++) tags_host[i] = (int64_t)t[i];
        }
        if (stamps_host) {
            std::vector<int32_t> t(lines);
            HIP_TRY(hipMemcpy(t.data(), stamps, lines * sizeof(int32_t), hipMemcpyDeviceToHost));
            for (uint64_t i = 0; i < lines; i++) stamps_host[i] = (int64_t)t[i];
        }
        return GIDS_OK;
    }
};

}  // namespace


// ---------------------------------------------------------------- sampler

struct gids_graph {
    uint64_t n_nodes = 0, n_edges = 0, n_words = 0;
    uint32_t id_bytes = 0;
    bool zero_copy = false;
    const int64_t* indptr = nullptr;     // device-visible
    const void* indices = nullptr;       // device-visible
    void* indptr_owned = nullptr;
    void* indices_owned = nullptr;
    uint64_t* bitmap = nullptr;
    uint32_t* blocksum = nullptr;        // bitmap scan
    uint32_t* blockoff = nullptr;
    uint32_t* hop_blocksum = nullptr;    // per-hop offsets
    uint32_t* hop_blockoff = nullptr;
    uint64_t hop_blocks_cap = 0;
    Ctl* ctl = nullptr;
    SamplerState* st = nullptr;
    void* frontier = nullptr;
    void* hop_out = nullptr;
    uint64_t cap_ids = 0;

    ~gids_graph() {
        (void)hipDeviceSynchronize();
        if (indptr_owned) (void)hipFree(indptr_owned);
        if (indices_owned) (void)hipFree(indices_owned);
        dev_free(bitmap); dev_free(blocksum); dev_free(blockoff); dev_free(hop_blocksum); dev_free(hop_blockoff);
        dev_free(ctl); dev_free(st);
        if (frontier) (void)hipFree(frontier);
        if (hop_out) (void)hipFree(hop_out);
    }

    int ensure(uint64_t ids, uint64_t hop_blocks) {
        if (ids > cap_ids) {
            HIP_TRY(hipDeviceSynchronize());
            if (frontier) (void)hipFree(frontier);
            if (hop_out) (void)hipFree(hop_out);
            frontier = hop_out = nullptr; cap_ids = 0;
            HIP_TRY(hipMalloc(&frontier, ids * id_bytes));
            HIP_TRY(hipMalloc(&hop_out, ids * id_bytes));
            cap_ids = ids;
        }
        if (hop_blocks > hop_blocks_cap) {
            HIP_TRY(hipDeviceSynchronize());
            dev_free(hop_blocksum); dev_free(hop_blockoff);
            hop_blocks_cap = 0;
            int rc;
            if ((rc = dev_alloc(&hop_blocksum, hop_blocks))) return rc;
            if ((rc = dev_alloc(&hop_blockoff, hop_blocks))) return rc;
            hop_blocks_cap = hop_blocks;
        }
        return GIDS_OK;
    }

    template <typename IdT>
    int sample(uint64_t seed, uint64_t batch, const uint32_t* fanouts, uint32_t n_layers, uint64_t n_seeds,
               const uint64_t* rank_table, uint64_t perm_mult, uint64_t perm_add, IdT* raw, uint32_t* n_raw_dev,
               hipStream_t s) {
        // bounds known on the host: hop l has at most n_seeds * f_0 * ... * f_(l-1) frontier nodes
        uint64_t front = std::min<uint64_t>(n_seeds, n_nodes), max_ids = std::max<uint64_t>(n_seeds, 1);
        for (uint32_t l = 0; l < n_layers; l++) {
            const uint64_t produced = front * fanouts[l];
            max_ids = std::max(max_ids, produced);
            front = std::min<uint64_t>(produced, n_nodes);
        }
        const uint64_t max_front = std::min<uint64_t>(max_ids, n_nodes);
        int rc = ensure(max_ids, (max_front + 255) / 256 + 1);
        if (rc) return rc;
        const uint64_t ks = sampler_mix(sampler_key(seed, 4) ^ batch);
        launch_seeds<IdT>(ks, n_seeds, n_nodes, rank_table, perm_mult, perm_add, raw, st, s);
        const IdT* hop_in = raw;                        // hop 0 expands the distinct seeds
        uint64_t in_upper = n_seeds;
        const uint32_t* in_count = nullptr;             // seeds: count known on the host
        front = std::min<uint64_t>(n_seeds, n_nodes);
        for (uint32_t l = 0; l < n_layers; l++) {
            // frontier = ascending distinct IDs of the previous hop's output
            launch_mark<IdT>(hop_in, in_upper, in_count, n_nodes, bitmap, ctl, s);
            launch_count(bitmap, n_words, blocksum, blockoff, ctl, &ctl->n_unique, s);
            launch_emit<IdT>(bitmap, n_words, n_nodes, blockoff, static_cast<IdT*>(frontier), nullptr, nullptr, true, ctl,
                             nullptr, s);
            const uint64_t kl = sampler_mix(sampler_mix(sampler_key(seed, 5) ^ batch) ^ (uint64_t)l);
            launch_hop<IdT>(static_cast<const IdT*>(frontier), &ctl->n_unique, front, indptr,
                            static_cast<const IdT*>(indices), fanouts[l], kl, hop_blocksum, hop_blockoff, raw,
                            static_cast<IdT*>(hop_out), st, s);
            hop_in = static_cast<const IdT*>(hop_out);
            in_upper = front * fanouts[l];
            in_count = &st->layer_count;
            front = std::min<uint64_t>(in_upper, n_nodes);
        }
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipMemcpyAsync(n_raw_dev, &st->n_raw, sizeof(uint32_t), hipMemcpyDeviceToDevice, s));
        return GIDS_OK;
    }
};

extern "C" {

const char* gids_last_error(void) { return g_err; }

int gids_store_create(uint64_t n_rows, uint32_t row_bytes, uint32_t id_bytes, void* host_ptr_or_null,
                      gids_store** out) {
    if (!out) return fail(GIDS_E_INVAL, "gids_store_create: out is NULL");
    *out = nullptr;
    if (n_rows == 0 || row_bytes == 0 || row_bytes % 16) return fail(GIDS_E_INVAL, "gids_store_create: row_bytes must be a positive multiple of 16 and n_rows > 0");
    if (id_bytes != 4 && id_bytes != 8) return fail(GIDS_E_INVAL, "gids_store_create: id_bytes must be 4 or 8");
    if (id_bytes == 4 && n_rows > 0x7FFFFFFFull) return fail(GIDS_E_INVAL, "gids_store_create: n_rows does not fit 4-byte IDs");
    if (n_rows > 0xFFFFFFFF00ull) return fail(GIDS_E_INVAL, "gids_store_create: n_rows too large");
    gids_store* st = new (std::nothrow) gids_store();
    if (!st) return fail(GIDS_E_NOMEM, "gids_store_create: out of host memory");
    st->n_rows = n_rows; st->row_bytes = row_bytes; st->id_bytes = id_bytes;
    if (hipGetDevice(&st->device) != hipSuccess) {
        (void)hipGetLastError();
        delete st;
        return fail(GIDS_E_HIP, "gids_store_create: no current device");
    }
    if (host_ptr_or_null) {
        st->host = host_ptr_or_null;
        hipError_t e = hipHostGetDevicePointer(&st->dev, host_ptr_or_null, 0);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            delete st;
            return fail(GIDS_E_HIP, "gids_store_create: host_ptr is not pinned, GPU-visible memory (%s)", hipGetErrorString(e));
        }
    } else {
        hipError_t e = hipHostMalloc(&st->host, n_rows * (uint64_t)row_bytes, hipHostMallocMapped);
        if (e == hipSuccess) e = hipHostGetDevicePointer(&st->dev, st->host, 0);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            if (st->host) (void)hipHostFree(st->host);
            delete st;
            return fail(GIDS_E_NOMEM, "gids_store_create: cannot pin %llu bytes of host memory (%s)",
                        (unsigned long long)(n_rows * (uint64_t)row_bytes), hipGetErrorString(e));
        }
        st->owned = true;
    }
    *out = st;
    return GIDS_OK;
}

void* gids_store_host_ptr(gids_store* store) { return store ? store->host : nullptr; }

int gids_store_destroy(gids_store* store) {
    if (!store) return GIDS_OK;
    if (store->owned && store->host) (void)hipHostFree(store->host);
    delete store;
    return GIDS_OK;
}

int gids_store_calibrate(gids_store* store, double* rows_per_s, double* overhead_s) {
    if (!store || !rows_per_s || !overhead_s) return fail(GIDS_E_INVAL, "gids_store_calibrate: NULL argument");
    const uint32_t n_small = 2048, n_large = 65536;
    char* out = nullptr;
    int rc = dev_alloc(&out, (uint64_t)n_large * store->row_bytes);
    if (rc) return rc;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    auto cleanup = [&]() {
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
        dev_free(out);
    };
    auto timed = [&](uint32_t n, int reps, double* best) -> int {
        *best = 1e30;
        for (int i = 0; i < reps + 1; i++) {                  // the first run warms up
            HIP_TRY(hipEventRecord(e0, nullptr));
            launch_calibrate(static_cast<const char*>(store->dev), store->n_rows, store->row_bytes, out, n, nullptr);
            HIP_TRY(hipEventRecord(e1, nullptr));
            HIP_TRY(hipEventSynchronize(e1));
            float ms = 0;
            HIP_TRY(hipEventElapsedTime(&ms, e0, e1));
            if (i && ms * 1e-3 < *best) *best = ms * 1e-3;
        }
        return GIDS_OK;
    };
    double t_small = 0, t_large = 0;
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    if (e != hipSuccess) { cleanup(); return fail(GIDS_E_HIP, "gids_store_calibrate: %s", hipGetErrorString(e)); }
    if ((rc = timed(n_small, 5, &t_small)) || (rc = timed(n_large, 3, &t_large))) { cleanup(); return rc; }
    cleanup();
    // t(n) = overhead + n / rate
    const double rate = (double)(n_large - n_small) / (t_large - t_small);
    *rows_per_s = rate;
    *overhead_s = t_small - n_small / rate;
    return GIDS_OK;
}

int gids_cache_create(gids_store* store, uint64_t lines, uint32_t ways, uint32_t line_bytes, uint32_t window_depth,
                      uint64_t accum_threshold, gids_cache** out) {
    if (!out) return fail(GIDS_E_INVAL, "gids_cache_create: out is NULL");
    *out = nullptr;
    if (!store) return fail(GIDS_E_INVAL, "gids_cache_create: store is NULL");
    if (!on_device(store->device)) return fail(GIDS_E_INVAL, "gids_cache_create: the current device is not the one the store was created on");
    if (ways == 0 || ways > 64 || (ways & (ways - 1))) return fail(GIDS_E_INVAL, "gids_cache_create: ways must be a power of two in [1, 64]");
    if (lines == 0 || lines % ways) return fail(GIDS_E_INVAL, "gids_cache_create: lines must be a positive multiple of ways");
    if (line_bytes < store->row_bytes || line_bytes % 16) return fail(GIDS_E_INVAL, "gids_cache_create: line_bytes must be a multiple of 16 and >= row_bytes");
    if (window_depth > 254) return fail(GIDS_E_INVAL, "gids_cache_create: window_depth must be <= 254");
    if (lines >= (1ull << 40) || accum_threshold >= (1ull << 31)) return fail(GIDS_E_INVAL, "gids_cache_create: lines or accum_threshold too large");
    gids_cache* c = store->id_bytes == 4 ? static_cast<gids_cache*>(new (std::nothrow) CacheT<int32_t>())
                                         : static_cast<gids_cache*>(new (std::nothrow) CacheT<int64_t>());
    if (!c) return fail(GIDS_E_NOMEM, "gids_cache_create: out of host memory");
    c->store = store; c->lines = lines; c->ways = ways; c->line_bytes = line_bytes; c->window = window_depth;
    c->threshold = accum_threshold; c->n_sets = lines / ways;
    c->lg_ways = 0;
    while ((1u << c->lg_ways) < ways) c->lg_ways++;
    const int rc = c->init();
    if (rc) { delete c; return rc; }
    // the static workspace's address on this device; a failure here only disables gids_gather_static
    if (static_workspace(store->device, &c->static_ws) != GIDS_OK) c->static_ws = nullptr;
    *out = c;
    return GIDS_OK;
}

int gids_cache_destroy(gids_cache* cache) {
    delete cache;
    return GIDS_OK;
}

#define CHECK_CACHE(c)                                                         \
    if (!(c)) return fail(GIDS_E_INVAL, "%s: cache is NULL", __func__);        \
    if (!on_device((c)->store->device)) return fail(GIDS_E_INVAL, "%s: the current device is not the one the store was created on", __func__); \
    (c)->poll_status();                                                        \
    if ((c)->sticky) return fail((c)->sticky, "%s: an earlier operation on this cache failed (%d)", __func__, (c)->sticky)

int gids_cache_reserve(gids_cache* cache, uint64_t max_ids) {
    CHECK_CACHE(cache);
    if (max_ids > 0xFFFFFFF0ull) return fail(GIDS_E_INVAL, "gids_cache_reserve: list too long");
    return cache->reserve(max_ids);
}

int gids_cpu_buffer_pin(gids_cache* cache, const void* ids_host, uint64_t n) {
    CHECK_CACHE(cache);
    return cache->pin(ids_host, n);
}

int gids_window_push(gids_cache* cache, const void* ids_dev, uint64_t n, void* stream) {
    CHECK_CACHE(cache);
    if (n > 0xFFFFFFF0ull) return fail(GIDS_E_INVAL, "gids_window_push: list too long");
    return cache->push(ids_dev, n, nullptr, static_cast<hipStream_t>(stream));
}

int gids_window_push_dev(gids_cache* cache, const void* ids_dev, uint64_t n_max, const uint32_t* n_dev, void* stream) {
    CHECK_CACHE(cache);
    if (n_max > 0xFFFFFFF0ull) return fail(GIDS_E_INVAL, "gids_window_push_dev: list too long");
    if (!n_dev) return fail(GIDS_E_INVAL, "gids_window_push_dev: n_dev is NULL");
    return cache->push(ids_dev, n_max, n_dev, static_cast<hipStream_t>(stream));
}

int gids_gather(gids_cache* cache, const void* ids_dev, uint64_t n, void* out_dev, uint64_t out_capacity_rows,
                void* unique_dev, void* inverse_dev, void* stream) {
    CHECK_CACHE(cache);
    if (n > 0xFFFFFFF0ull) return fail(GIDS_E_INVAL, "gids_gather: list too long");
    return cache->gather(ids_dev, n, out_dev, out_capacity_rows, unique_dev, inverse_dev, false, static_cast<hipStream_t>(stream));
}

int gids_gather_static(gids_cache* cache, const void* ids_dev, uint64_t n, void* out_dev, uint64_t out_capacity_rows,
                       void* unique_dev, void* stream) {
    CHECK_CACHE(cache);
    if (n > STATIC_MAX_IDS) return fail(GIDS_E_INVAL, "gids_gather_static: a list of %llu IDs exceeds the static workspace (GIDS_STATIC_MAX_IDS = %llu)", (unsigned long long)n, (unsigned long long)STATIC_MAX_IDS);
    if (!cache->static_ws) return fail(GIDS_E_HIP, "gids_gather_static: the static workspace of this device could not be located when the cache was created");
    return cache->gather(ids_dev, n, out_dev, out_capacity_rows, unique_dev, nullptr, true, static_cast<hipStream_t>(stream));
}

int gids_cache_set_policy(gids_cache* cache, int policy, uint64_t seed) {
    CHECK_CACHE(cache);
    if (policy != GIDS_POLICY_LRU && policy != GIDS_POLICY_RANDOM) return fail(GIDS_E_INVAL, "gids_cache_set_policy: unknown policy %d", policy);
    if (cache->seq) return fail(GIDS_E_INVAL, "gids_cache_set_policy: call before the first gather");
    cache->policy = (uint32_t)policy;
    cache->policy_key = sampler_mix(seed + 8ull * 0x9E3779B97F4A7C15ull);
    return GIDS_OK;
}

int gids_cache_set_accum_mode(gids_cache* cache, int mode) {
    CHECK_CACHE(cache);
    if (mode != GIDS_ACCUM_FIXED && mode != GIDS_ACCUM_ADAPTIVE) return fail(GIDS_E_INVAL, "gids_cache_set_accum_mode: unknown mode %d", mode);
    if (!cache->threshold) return fail(GIDS_E_INVAL, "gids_cache_set_accum_mode: the cache was created without an accumulator (accum_threshold == 0)");
    if (cache->seq) return fail(GIDS_E_INVAL, "gids_cache_set_accum_mode: call before the first gather");
    cache->accum_mode = mode;
    return GIDS_OK;
}

int gids_cache_set_group_dedup(gids_cache* cache, int on) {
    CHECK_CACHE(cache);
    if (!cache->threshold) return fail(GIDS_E_INVAL, "gids_cache_set_group_dedup: the cache was created without an accumulator (accum_threshold == 0)");
    if (cache->open_batches) return fail(GIDS_E_INVAL, "gids_cache_set_group_dedup: a group of minibatches is open (call gids_flush first)");
    cache->group_dedup = on != 0;
    return GIDS_OK;
}

int gids_cache_set_rows_per_line(gids_cache* cache, uint32_t rows) {
    CHECK_CACHE(cache);
    if (rows < 1) return fail(GIDS_E_INVAL, "gids_cache_set_rows_per_line: rows must be >= 1");
    if ((uint64_t)rows * cache->store->row_bytes > cache->line_bytes) return fail(GIDS_E_INVAL, "gids_cache_set_rows_per_line: %u rows of %u bytes do not fit a line of %u bytes", rows, cache->store->row_bytes, cache->line_bytes);
    if (cache->threshold && rows > 1) return fail(GIDS_E_INVAL, "gids_cache_set_rows_per_line: not available together with the accumulator");
    if (cache->seq || cache->window_count()) return fail(GIDS_E_INVAL, "gids_cache_set_rows_per_line: call before the first push or gather");
    cache->rows_per_line = rows;
    return GIDS_OK;
}

int gids_gather_many(gids_cache* cache, uint32_t k, const void* const* push_ids_dev, const uint64_t* push_n,
                     void* const* out_dev, const uint64_t* out_capacity_rows, void* const* unique_dev, void* push_stream,
                     void* stream) {
    CHECK_CACHE(cache);
    if (push_ids_dev && !push_n) return fail(GIDS_E_INVAL, "gids_gather_many: push_n is NULL");
    return cache->gather_many(k, push_ids_dev, push_n, out_dev, out_capacity_rows, unique_dev,
                              static_cast<hipStream_t>(push_stream), static_cast<hipStream_t>(stream));
}

int gids_flush(gids_cache* cache, void* stream) {
    CHECK_CACHE(cache);
    return cache->flush(static_cast<hipStream_t>(stream));
}

int gids_stats_read(gids_cache* cache, uint64_t seq, gids_stats* stats) {
    if (!cache || !stats) return fail(GIDS_E_INVAL, "gids_stats_read: NULL argument");
    if (seq >= cache->seq || seq + STATS_RING < cache->seq) return fail(GIDS_E_INVAL, "gids_stats_read: gather %llu is not available", (unsigned long long)seq);
    const int r = (int)(seq % STATS_RING);
    const int er = cache->ev_of[r];
    if (cache->pipelined) HIP_TRY(hipEventSynchronize(cache->ev_meta[er]));
    HIP_TRY(hipEventSynchronize(cache->events[er]));
    const StatsRec rec = cache->ring_host[r];
    if (rec.seq != seq) return fail(GIDS_E_INVAL, "gids_stats_read: record of gather %llu was overwritten", (unsigned long long)seq);
    stats->seq = rec.seq; stats->n_unique = rec.n_unique; stats->n_hit = rec.n_hit; stats->n_cpu_hit = rec.n_cpu_hit;
    stats->n_miss = rec.n_miss; stats->n_bypass = rec.n_bypass; stats->n_pending = rec.n_pending;
    stats->flushed = rec.flushed; stats->status = rec.status; stats->n_line_fills = rec.n_line_fills;
    stats->n_cpu_again = rec.n_cpu_again;
    if (rec.status) {
        cache->sticky = rec.status;
        return fail(rec.status, "gather %llu failed on the device with code %d", (unsigned long long)seq, rec.status);
    }
    return GIDS_OK;
}

int gids_profile_enable(gids_cache* cache, int on) {
    if (!cache) return fail(GIDS_E_INVAL, "gids_profile_enable: cache is NULL");
    cache->profile = on != 0;
    return GIDS_OK;
}

int gids_profile_read(gids_cache* cache, uint64_t seq, float* ms3) {
    if (!cache || !ms3) return fail(GIDS_E_INVAL, "gids_profile_read: NULL argument");
    if (seq >= cache->seq || seq + STATS_RING < cache->seq) return fail(GIDS_E_INVAL, "gids_profile_read: gather %llu is not available", (unsigned long long)seq);
    const int r = (int)(seq % STATS_RING);
    if (!cache->prof_valid[r]) return fail(GIDS_E_INVAL, "gids_profile_read: gather %llu was not profiled", (unsigned long long)seq);
    HIP_TRY(hipEventSynchronize(cache->prof_events[r][2]));
    HIP_TRY(hipEventSynchronize(cache->prof_events[r][4]));
    HIP_TRY(hipEventElapsedTime(&ms3[0], cache->prof_events[r][0], cache->prof_events[r][1]));
    HIP_TRY(hipEventElapsedTime(&ms3[1], cache->prof_events[r][1], cache->prof_events[r][2]));
    HIP_TRY(hipEventElapsedTime(&ms3[2], cache->prof_events[r][3], cache->prof_events[r][4]));
    return GIDS_OK;
}

uint64_t gids_cache_gathers(const gids_cache* cache) { return cache ? cache->seq : 0; }

void gids_cache_many_calls(const gids_cache* cache, uint64_t* merged_kernels, uint64_t* per_step_kernels) {
    if (merged_kernels) *merged_kernels = cache ? cache->many_fast_calls : 0;
    if (per_step_kernels) *per_step_kernels = cache ? cache->many_slow_calls : 0;
}

int gids_cache_snapshot(gids_cache* cache, int64_t* tags_host, int64_t* stamps_host) {
    if (!cache) return fail(GIDS_E_INVAL, "gids_cache_snapshot: cache is NULL");
    return cache->snapshot(tags_host, stamps_host);
}


int gids_graph_create(uint64_t n_nodes, const int64_t* indptr_host, const void* indices_host, uint32_t id_bytes,
                      int zero_copy, gids_graph** out) {
    if (!out) return fail(GIDS_E_INVAL, "gids_graph_create: out is NULL");
    *out = nullptr;
    if (!indptr_host || !indices_host || n_nodes == 0) return fail(GIDS_E_INVAL, "gids_graph_create: NULL or empty graph");
    if (id_bytes != 4 && id_bytes != 8) return fail(GIDS_E_INVAL, "gids_graph_create: id_bytes must be 4 or 8");
    if (id_bytes == 4 && n_nodes > 0x7FFFFFFFull) return fail(GIDS_E_INVAL, "gids_graph_create: n_nodes does not fit 4-byte IDs");
    if (indptr_host[0] != 0 || indptr_host[n_nodes] < 0) return fail(GIDS_E_INVAL, "gids_graph_create: indptr must start at 0");
    gids_graph* g = new (std::nothrow) gids_graph();
    if (!g) return fail(GIDS_E_NOMEM, "gids_graph_create: out of host memory");
    g->n_nodes = n_nodes; g->n_edges = (uint64_t)indptr_host[n_nodes]; g->id_bytes = id_bytes; g->zero_copy = zero_copy != 0;
    g->n_words = (n_nodes + 63) / 64;
    auto bail = [&](int rc) { delete g; return rc; };
    if (zero_copy) {
        void *p = nullptr, *q = nullptr;
        hipError_t e = hipHostGetDevicePointer(&p, const_cast<int64_t*>(indptr_host), 0);
        if (e == hipSuccess) e = hipHostGetDevicePointer(&q, const_cast<void*>(indices_host), 0);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return bail(fail(GIDS_E_HIP, "gids_graph_create: zero_copy needs arrays allocated with hipHostMalloc (%s)", hipGetErrorString(e)));
        }
        g->indptr = static_cast<const int64_t*>(p); g->indices = q;
    } else {
        hipError_t e = hipMalloc(&g->indptr_owned, (n_nodes + 1) * sizeof(int64_t));
        if (e == hipSuccess) e = hipMalloc(&g->indices_owned, std::max<uint64_t>(g->n_edges, 1) * id_bytes);
        if (e == hipSuccess) e = hipMemcpy(g->indptr_owned, indptr_host, (n_nodes + 1) * sizeof(int64_t), hipMemcpyHostToDevice);
        if (e == hipSuccess && g->n_edges) e = hipMemcpy(g->indices_owned, indices_host, g->n_edges * id_bytes, hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return bail(fail(e == hipErrorOutOfMemory ? GIDS_E_NOMEM : GIDS_E_HIP, "gids_graph_create: %s", hipGetErrorString(e)));
        }
        g->indptr = static_cast<const int64_t*>(g->indptr_owned); g->indices = g->indices_owned;
    }
    int rc;
    if ((rc = dev_alloc(&g->bitmap, g->n_words))) return bail(rc);
    const uint32_t nb = scan_blocks(g->n_words);
    if ((rc = dev_alloc(&g->blocksum, nb))) return bail(rc);
    if ((rc = dev_alloc(&g->blockoff, nb))) return bail(rc);
    if ((rc = dev_alloc(&g->ctl, 1))) return bail(rc);
    if ((rc = dev_alloc(&g->st, 1))) return bail(rc);
    hipError_t e = hipMemset(g->bitmap, 0, g->n_words * sizeof(uint64_t));
    if (e == hipSuccess) e = hipMemset(g->ctl, 0, sizeof(Ctl));
    if (e == hipSuccess) e = hipMemset(g->st, 0, sizeof(SamplerState));
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) return bail(fail(GIDS_E_HIP, "gids_graph_create: %s", hipGetErrorString(e)));
    *out = g;
    return GIDS_OK;
}

int gids_graph_destroy(gids_graph* graph) {
    delete graph;
    return GIDS_OK;
}

uint64_t gids_sample_capacity(const uint32_t* fanouts, uint32_t n_layers, uint64_t n_seeds) {
    uint64_t total = n_seeds, width = n_seeds;
    for (uint32_t l = 0; l < n_layers; l++) {
        width *= fanouts ? fanouts[l] : 0;
        total += width;
    }
    return total;
}

int gids_sample(gids_graph* graph, uint64_t seed, uint64_t batch, const uint32_t* fanouts, uint32_t n_layers,
                uint64_t n_seeds, const uint64_t* rank_table_dev, uint64_t perm_mult, uint64_t perm_add, void* raw_dev,
                uint64_t raw_capacity, uint32_t* n_raw_dev, void* stream) {
    if (!graph || !raw_dev || !n_raw_dev) return fail(GIDS_E_INVAL, "gids_sample: NULL argument");
    if (n_layers > 8 || (n_layers && !fanouts)) return fail(GIDS_E_INVAL, "gids_sample: at most 8 layers");
    for (uint32_t l = 0; l < n_layers; l++)
        if (fanouts[l] < 1 || fanouts[l] > 64) return fail(GIDS_E_INVAL, "gids_sample: fanouts must be in [1, 64]");
    const uint64_t need = gids_sample_capacity(fanouts, n_layers, n_seeds);
    if (need > 0xFFFFFFF0ull) return fail(GIDS_E_INVAL, "gids_sample: minibatch too large");
    if (raw_capacity < need) return fail(GIDS_E_SPACE, "gids_sample: raw_dev must hold %llu IDs (gids_sample_capacity)", (unsigned long long)need);
    if (rank_table_dev && graph->n_nodes >= (1ull << 31)) return fail(GIDS_E_INVAL, "gids_sample: ranked seeds need n_nodes < 2^31");
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (graph->id_bytes == 4)
        return graph->sample<int32_t>(seed, batch, fanouts, n_layers, n_seeds, rank_table_dev, perm_mult, perm_add,
                                      static_cast<int32_t*>(raw_dev), n_raw_dev, s);
    return graph->sample<int64_t>(seed, batch, fanouts, n_layers, n_seeds, rank_table_dev, perm_mult, perm_add,
                                  static_cast<int64_t*>(raw_dev), n_raw_dev, s);
}

int gids_graph_visit_scores(gids_graph* graph, const uint32_t* fanouts, uint32_t n_layers, uint64_t n_seeds,
                            uint64_t* scores_dev, void* stream) {
    if (!graph || !scores_dev) return fail(GIDS_E_INVAL, "gids_graph_visit_scores: NULL argument");
    if (n_layers > 8 || (n_layers && !fanouts)) return fail(GIDS_E_INVAL, "gids_graph_visit_scores: at most 8 layers");
    for (uint32_t l = 0; l < n_layers; l++)
        if (fanouts[l] < 1 || fanouts[l] > 64) return fail(GIDS_E_INVAL, "gids_graph_visit_scores: fanouts must be in [1, 64]");
    if (n_seeds > (1ull << 30)) return fail(GIDS_E_INVAL, "gids_graph_visit_scores: n_seeds too large");
    uint64_t *cur = nullptr, *nxt = nullptr;
    int rc;
    if ((rc = dev_alloc(&cur, graph->n_nodes))) return rc;
    if ((rc = dev_alloc(&nxt, graph->n_nodes))) { dev_free(cur); return rc; }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (graph->id_bytes == 4)
        launch_visit_scores<int32_t>(graph->indptr, static_cast<const int32_t*>(graph->indices), graph->n_nodes, fanouts,
                                     n_layers, n_seeds, cur, nxt, scores_dev, s);
    else
        launch_visit_scores<int64_t>(graph->indptr, static_cast<const int64_t*>(graph->indices), graph->n_nodes, fanouts,
                                     n_layers, n_seeds, cur, nxt, scores_dev, s);
    hipError_t e = hipStreamSynchronize(s);                  // the scratch arrays go away with the call
    dev_free(cur); dev_free(nxt);
    if (e != hipSuccess) return fail(GIDS_E_HIP, "gids_graph_visit_scores: %s", hipGetErrorString(e));
    return GIDS_OK;
}

int gids_graph_reverse_pagerank(gids_graph* graph, uint32_t damping_q16, uint32_t n_iters, uint64_t* scores_dev,
                                void* stream) {
    if (!graph || !scores_dev) return fail(GIDS_E_INVAL, "gids_graph_reverse_pagerank: NULL argument");
    if (damping_q16 > 65536u || n_iters > 10000u) return fail(GIDS_E_INVAL, "gids_graph_reverse_pagerank: damping_q16 must be <= 65536 and n_iters <= 10000");
    uint64_t* scratch = nullptr;
    int rc;
    if ((rc = dev_alloc(&scratch, graph->n_nodes))) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (graph->id_bytes == 4)
        launch_reverse_pagerank<int32_t>(graph->indptr, static_cast<const int32_t*>(graph->indices), graph->n_nodes,
                                         damping_q16, n_iters, scratch, scores_dev, s);
    else
        launch_reverse_pagerank<int64_t>(graph->indptr, static_cast<const int64_t*>(graph->indices), graph->n_nodes,
                                         damping_q16, n_iters, scratch, scores_dev, s);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(s);        // the scratch array goes away with the call
    dev_free(scratch);
    if (e != hipSuccess) return fail(GIDS_E_HIP, "gids_graph_reverse_pagerank: %s", hipGetErrorString(e));
    return GIDS_OK;
}

double gids_accum_threshold(double iops_peak, double t_initial, double t_termination, double ratio, int n_ssd) {
    // N = IOPS_achieved * (Ti + Ts + Tt) * n_ssd with Ts = N / (IOPS_peak * n_ssd), at IOPS_achieved = ratio * IOPS_peak
    if (!(ratio > 0.0) || !(ratio < 1.0) || n_ssd < 1) return -1.0;
    const double busy = iops_peak * (double)n_ssd;
    return ratio * busy * (t_initial + t_termination) / (1.0 - ratio);
}

}  // extern "C"
