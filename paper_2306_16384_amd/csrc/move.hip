// Row movement of the feature gather (GIDS paper, Section 2.2.3 for the
// gather, Section 3.2 for batching accesses across minibatches, Section 3.3
// for rows redirected to the CPU buffer).
//
//   move      one group of lanes per output row, 16 bytes per lane per access:
//             a hit copies cache line -> output (HBM -> HBM); a CPU-buffer hit
//             copies pinned host row -> output; a miss reads the host store row
//             once and writes it to the output and, when a victim line was
//             found, to that line (the "line fill").  Tags were published by
//             the commit kernel before; only bytes move here.
//   queue     the accumulator's variant: nothing moves; every row of the
//             minibatch becomes an operation in the lists of the open group.
//   group     when a group of minibatches closes, its rows move in two
//   mover     launches (link rows and plain hit copies; then the copies that
//             depend on them).
//   finalize  publishes the minibatch's counters to host-visible memory and
//             advances the minibatch stamp.
#include <cstdlib>

#include "gids_dev.h"
#include "gather_dev.h"

namespace gids {

namespace {

constexpr int MV_THREADS = 256;
constexpr int MV_UNROLL = 4;

// Rows are streamed: read once, written once or twice, far larger in total than
// L2 or the memory-side cache, so every access carries the non-temporal hint.
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

template <int G>
__device__ __forceinline__ void copy_row(const v4u* __restrict__ src, v4u* __restrict__ dst,
                                         v4u* __restrict__ dst2, uint32_t row_u4, uint32_t sub) {
    for (uint32_t k0 = 0; k0 < row_u4; k0 += G * MV_UNROLL) {
        v4u buf[MV_UNROLL];
#pragma unroll
        for (int u = 0; u < MV_UNROLL; u++) {
            const uint32_t k = k0 + u * G + sub;
            if (k < row_u4) buf[u] = __builtin_nontemporal_load(src + k);
        }
#pragma unroll
        for (int u = 0; u < MV_UNROLL; u++) {
            const uint32_t k = k0 + u * G + sub;
            if (k < row_u4) {
                __builtin_nontemporal_store(buf[u], dst + k);
                if (dst2) __builtin_nontemporal_store(buf[u], dst2 + k);
            }
        }
    }
}

// position of the n-th (0-based) set bit of mask, or 64 when there are fewer
__device__ __forceinline__ uint32_t nth_set_bit(uint64_t mask, uint32_t n) {
    for (uint32_t i = 0; i < n; i++) mask &= mask - 1;
    return mask ? (uint32_t)(__ffsll((unsigned long long)mask) - 1) : 64u;
}

// The first `link_blocks` workgroups move the rows that cross the host link
// (CPU-buffer rows, store rows), the others the rows that stay in HBM (hits).
// About fifty persistent workgroups (one row in flight per wave) bring the
// link within half a percent of what a hundred reach; every request beyond
// what the link can carry only queues in front of the memory traffic of every
// other kernel on the GPU (the next minibatch's classification, the consumer
// of the previous one), which a hundred slow down several times over.  HBM
// wants thousands of waves; both halves run concurrently.
// A wave reads CH plan entries with one coalesced load, ballots which of them
// belong to its half, and then moves those rows 64 / G at a time, so scanning
// past the other half's rows costs one load per CH rows.
template <typename IdT, int G>
__global__ __launch_bounds__(MV_THREADS) void move_kernel(CacheView<IdT> c, const IdT* __restrict__ unique,
                                                          BatchHdr* __restrict__ hdr,
                                                          const uint64_t* __restrict__ plan, char* __restrict__ out,
                                                          IdT* __restrict__ unique_out, uint32_t link_blocks,
                                                          uint32_t link_ch, uint32_t hbm_ch, uint32_t link_spread) {
    if (!hdr->ok) return;
    const uint32_t n_u = hdr->n_u;
    const uint32_t row_u4 = c.row_bytes >> 4;
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t sub = lane % G, grp = lane / G;
    constexpr uint32_t PER_ITER = 64 / G;                     // rows a wave moves at once
    const bool link_role = blockIdx.x < link_blocks;
    uint32_t ch = link_role ? link_ch : hbm_ch;               // plan entries a wave scans per step
    const uint32_t role_block = link_role ? blockIdx.x : blockIdx.x - link_blocks;
    const uint32_t role_blocks = link_role ? link_blocks : gridDim.x - link_blocks;
    const uint64_t wave0 = ((uint64_t)role_block * MV_THREADS + threadIdx.x) >> 6;
    const uint64_t n_waves = ((uint64_t)role_blocks * MV_THREADS) >> 6;
    // HBM half: chunk = wave index, strided.  Link half: the persistent waves draw chunks from a counter, so
    // that none is left with a long tail of slow rows while the others have run out of work.
    // The host sized link_ch for the longest list this call may hold; with the real count known here the
    // chunks shrink until every link wave can expect a few of them, which is what evens out the finish.
    if (link_role)
        while (ch > 4 && n_u / ch < link_spread * n_waves) ch >>= 1;
    uint64_t base = wave0 * ch;
    for (;;) {
        if (link_role) {
            uint32_t chunk = 0;
            if (lane == 0) chunk = atomicAdd(&hdr->next_chunk, 1u);
            base = (uint64_t)__shfl(chunk, 0) * ch;
        }
        if (base >= n_u) break;
        const uint64_t jl = base + lane;
        uint64_t e = 0, v = 0;
        bool mine = false;
        if (lane < ch && jl < n_u) {
            e = plan[jl];
            v = (uint64_t)unique[jl];
            mine = ((e >> PLAN_SHIFT) != PLAN_HIT) == link_role;
            if (!link_role && unique_out) unique_out[jl] = (IdT)v;   // the HBM half sees every j exactly once
        }
        uint64_t todo = __ballot(mine);
        while (todo) {
            const uint32_t pick = nth_set_bit(todo, grp);
#pragma unroll
            for (uint32_t i = 0; i < PER_ITER; i++) todo &= todo - 1;    // (clearing bits of 0 leaves 0)
            const uint64_t e_p = __shfl(e, (int)(pick & 63));
            const uint64_t v_p = __shfl(v, (int)(pick & 63));
            if (pick == 64u) continue;
            const uint64_t kind = e_p >> PLAN_SHIFT, idx = e_p & PLAN_INDEX_MASK;
            const uint64_t rpl = c.rows_per_line;
            const char* src;
            char* line = nullptr;
            if (kind == PLAN_HIT) {
                src = c.cache_data + idx * c.line_bytes;
                if (rpl > 1) src += (v_p - store_line_of(c, v_p) * rpl) * c.row_bytes;   // the row's place in its line
            } else if (kind == PLAN_CPU) {
                src = c.cpubuf + idx * c.row_bytes;
            } else {
                src = c.store + v_p * c.row_bytes;
                if (kind == PLAN_INSTALL) line = c.cache_data + idx * c.line_bytes;
            }
            v4u* dst = reinterpret_cast<v4u*>(out + (base + pick) * c.row_bytes);
            if (rpl == 1 || !line) {
                copy_row<G>(reinterpret_cast<const v4u*>(src), dst, reinterpret_cast<v4u*>(line), row_u4, sub);
            } else {
                // several rows per line: the requested row to the output, then the whole store line (clipped at
                // the table's end) into the cache line
                copy_row<G>(reinterpret_cast<const v4u*>(src), dst, nullptr, row_u4, sub);
                const uint64_t first = store_line_of(c, v_p) * rpl;
                const uint64_t rows = first + rpl <= c.n_rows ? rpl : c.n_rows - first;
                copy_row<G>(reinterpret_cast<const v4u*>(c.store + first * c.row_bytes), reinterpret_cast<v4u*>(line),
                            nullptr, (uint32_t)(rows * row_u4), sub);
            }
        }
        if (!link_role) base += n_waves * ch;
    }
}

// The accumulator's variant of the row mover: one plan entry per lane, appended to the open group's lists
// (queue_entry).
template <typename IdT>
__global__ __launch_bounds__(MV_THREADS) void queue_kernel(CacheView<IdT> c, AccumView a, uint32_t group,
                                                           const IdT* __restrict__ unique,
                                                           const BatchHdr* __restrict__ hdr,
                                                           const uint64_t* __restrict__ plan, char* __restrict__ out,
                                                           IdT* __restrict__ unique_out) {
    if (!hdr->ok) return;
    const uint32_t n_u = hdr->n_u;
    const uint32_t lane = threadIdx.x & 63;
    const uint64_t wave0 = ((uint64_t)blockIdx.x * MV_THREADS + threadIdx.x) >> 6;
    const uint64_t n_waves = ((uint64_t)gridDim.x * MV_THREADS) >> 6;
    for (uint64_t base = wave0 * 64; base < n_u; base += n_waves * 64) {
        const uint64_t j = base + lane;
        const bool valid = j < n_u;
        uint64_t e = 0, v = 0;
        if (valid) {
            e = plan[j];
            v = (uint64_t)unique[j];
        }
        queue_entry(c, a, group, valid, j, e, v, out, unique_out, true);
    }
}

// What is left of a gather once its victims are chosen, in one launch: the commit (tag and stamp of every
// line a miss was given, the miss mask back to zero), with the accumulator the queueing of every row, and,
// by the last workgroup to finish, the header the row mover reads and the counters.  After this kernel the
// next minibatch may be classified, whether or not the rows of this one have moved yet.
template <typename IdT>
__global__ __launch_bounds__(MV_THREADS) void settle_kernel(CacheView<IdT> c, AccumView a, uint32_t group, int accum,
                                                            const IdT* __restrict__ unique,
                                                            const uint32_t* __restrict__ n_u_ptr,
                                                            const uint64_t* __restrict__ plan, BatchHdr* hdr,
                                                            char* __restrict__ out, IdT* __restrict__ unique_out,
                                                            StatsRec* rec, uint64_t seq) {
    __shared__ uint32_t is_last;
    Ctl* ctl = c.ctl;
    const bool ok = ld_agent(&ctl->error) == 0;              // (set by earlier kernels; this one only on a list overflow)
    const uint32_t n_all = *n_u_ptr;
    const uint32_t n_u = ok ? n_all : 0;
    const uint32_t stamp = ctl->stamp;
    const bool any_miss = ctl->cnt_miss != 0;                // final: the probe has ended
    const uint32_t lane = threadIdx.x & 63;
    const uint64_t wave0 = ((uint64_t)blockIdx.x * MV_THREADS + threadIdx.x) >> 6;
    const uint64_t n_waves = ((uint64_t)gridDim.x * MV_THREADS) >> 6;
    if (any_miss || accum) {
        for (uint64_t base = wave0 * 64; base < n_u; base += n_waves * 64) {
            const uint64_t j = base + lane;
            const bool valid = j < n_u;
            uint64_t e = 0, v = 0;
            if (valid) {
                e = plan[j];
                v = (uint64_t)unique[j];
                const uint64_t kind = e >> PLAN_SHIFT;
                if (any_miss && kind >= PLAN_INSTALL) {
                    const uint64_t b = store_line_of(c, v);
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
            if (accum) queue_entry(c, a, group, valid, j, e, v, out, unique_out, true);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();
        is_last = atomicAdd(&ctl->ticket_cls, 1u) == gridDim.x - 1;
    }
    __syncthreads();
    if (!is_last || threadIdx.x != 0) return;
    __threadfence();
    const bool good = ld_agent(&ctl->error) == 0;
    hdr->ok = good ? 1u : 0u;
    hdr->n_u = good ? n_all : 0u;
    hdr->stamp = stamp;
    hdr->next_chunk = 0;
    ctl->ticket_cls = 0;
    publish_stats(ctl, rec, seq, n_all, accum);
}

// The group mover, first launch: the fills and the rcopies of one closed group.  Shaped like the row mover:
// the first `link_blocks` workgroups are persistent and draw chunks of fills from a counter (rows that cross
// the host link), the next `hbm_blocks` copy cache lines to output rows; when a caller asked for distinct-ID
// lists, one more workgroup per minibatch of the group copies its list from the group's staging buffer to the
// caller's buffer (as 32-bit words).
template <int G>
__global__ __launch_bounds__(MV_THREADS) void group_move_kernel(Ctl* ctl, const FillOp* __restrict__ fills,
                                                                const CopyOp* __restrict__ rcopies,
                                                                char* __restrict__ cache_data, uint32_t line_bytes,
                                                                uint32_t row_bytes, uint32_t par, uint32_t link_blocks,
                                                                uint32_t hbm_blocks, uint32_t link_ch,
                                                                uint32_t link_spread, UniqCopies u,
                                                                const uint32_t* __restrict__ stage, uint32_t id_words) {
    if (blockIdx.x >= link_blocks + hbm_blocks) {
        const uint32_t i = blockIdx.x - link_blocks - hbm_blocks;
        uint32_t* __restrict__ dst = static_cast<uint32_t*>(u.dst[i]);
        if (!dst) return;
        const uint32_t* __restrict__ src = stage + u.src_entry[i] * id_words;
        const uint64_t n = (uint64_t)ctl->grp_nu[par][i] * id_words;
        for (uint64_t j = threadIdx.x; j < n; j += MV_THREADS) dst[j] = src[j];
        return;
    }
    const uint32_t row_u4 = row_bytes >> 4;
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t sub = lane % G, grp = lane / G;
    constexpr uint32_t PER_ITER = 64 / G;                     // rows a wave moves at once
    // A wave reads up to 64 operations with one coalesced load (lane i holds operation base + i) and then
    // moves their rows PER_ITER at a time, each group of G lanes taking its operation from the holder's lane.
    if (blockIdx.x < link_blocks) {
        const uint32_t n = ctl->q_fill[par];
        const uint64_t n_waves = ((uint64_t)link_blocks * MV_THREADS) >> 6;
        uint32_t ch = link_ch;
        while (ch > 4 && n / ch < link_spread * n_waves) ch >>= 1;
        if (ch < PER_ITER) ch = PER_ITER;
        for (;;) {
            uint32_t chunk = 0;
            if (lane == 0) chunk = atomicAdd(&ctl->q_chunk[par], 1u);
            const uint64_t base = (uint64_t)__shfl(chunk, 0) * ch;
            if (base >= n) break;
            FillOp op;
            op.src = nullptr; op.dst_out = nullptr; op.dst_line = NO_LINE;
            if (lane < ch && base + lane < n) op = fills[base + lane];
            const uint32_t m = (uint32_t)(n - base < ch ? n - base : ch);
            for (uint32_t i0 = 0; i0 < m; i0 += PER_ITER) {
                const uint32_t i = i0 + grp;
                const uint64_t src = __shfl((uint64_t)op.src, (int)(i & 63));
                const uint64_t dst = __shfl((uint64_t)op.dst_out, (int)(i & 63));
                const uint64_t dl = __shfl(op.dst_line, (int)(i & 63));
                if (i >= m || !src) continue;                 // (a place that was taken and not needed)
                char* line = dl == NO_LINE ? nullptr : cache_data + dl * line_bytes;
                copy_row<G>(reinterpret_cast<const v4u*>(src), reinterpret_cast<v4u*>(dst),
                            reinterpret_cast<v4u*>(line), row_u4, sub);
            }
        }
    } else {
        const uint32_t n = ctl->q_rcopy[par];
        const uint64_t wave0 = ((uint64_t)(blockIdx.x - link_blocks) * MV_THREADS + threadIdx.x) >> 6;
        const uint64_t n_waves = ((uint64_t)hbm_blocks * MV_THREADS) >> 6;
        constexpr uint32_t CH = 16;                           // operations a wave takes per step
        for (uint64_t base = wave0 * CH; base < n; base += n_waves * CH) {
            CopyOp op;
            op.src = nullptr; op.dst = nullptr;
            if (lane < CH && base + lane < n) op = rcopies[base + lane];
            const uint32_t m = (uint32_t)(n - base < CH ? n - base : CH);
            for (uint32_t i0 = 0; i0 < m; i0 += PER_ITER) {
                const uint32_t i = i0 + grp;
                const uint64_t src = __shfl((uint64_t)op.src, (int)(i & 63));
                const uint64_t dst = __shfl((uint64_t)op.dst, (int)(i & 63));
                if (i >= m || !dst) continue;                 // (a place that was taken and not needed)
                copy_row<G>(reinterpret_cast<const v4u*>(src), reinterpret_cast<v4u*>(dst), nullptr, row_u4, sub);
            }
        }
    }
}

// second launch: the copies that had to wait for the first.  The last workgroup to finish empties the group's
// lists: the next group of this parity starts appending only after this kernel has ended.
template <int G>
__global__ __launch_bounds__(MV_THREADS) void group_copy_kernel(Ctl* ctl, const CopyOp* __restrict__ wcopies,
                                                                uint32_t row_bytes, uint32_t par) {
    const uint32_t n = ctl->q_wcopy[par];
    const uint32_t row_u4 = row_bytes >> 4;
    const uint32_t sub = threadIdx.x % G;
    const uint64_t g0 = ((uint64_t)blockIdx.x * MV_THREADS + threadIdx.x) / G;
    const uint64_t n_groups = (uint64_t)gridDim.x * MV_THREADS / G;
    for (uint64_t k = g0; k < n; k += n_groups) {
        const CopyOp op = wcopies[k];
        if (!op.dst) continue;                                // cancelled: its line was given away again
        copy_row<G>(reinterpret_cast<const v4u*>(op.src), reinterpret_cast<v4u*>(op.dst), nullptr, row_u4, sub);
    }
    __syncthreads();                                          // every thread of the block has read n
    if (threadIdx.x == 0) {
        __threadfence();
        if (atomicAdd(&ctl->ticket_flush, 1u) == gridDim.x - 1) {
            ctl->q_fill[par] = ctl->q_rcopy[par] = ctl->q_wcopy[par] = ctl->q_chunk[par] = 0;
            ctl->ticket_flush = 0;
        }
    }
}

// Link calibration: `n` rows of the host table, picked by a hash of their index, copied to a scratch
// buffer with the link half's shape (persistent workgroups, one wavefront per row).
template <int G>
__global__ __launch_bounds__(MV_THREADS) void calibrate_kernel(const char* __restrict__ store, uint64_t store_rows,
                                                               uint32_t row_bytes, char* __restrict__ out, uint32_t n) {
    const uint32_t row_u4 = row_bytes >> 4;
    const uint32_t sub = threadIdx.x % G;
    const uint64_t g0 = ((uint64_t)blockIdx.x * MV_THREADS + threadIdx.x) / G;
    const uint64_t n_groups = (uint64_t)gridDim.x * MV_THREADS / G;
    for (uint64_t j = g0; j < n; j += n_groups) {
        uint64_t z = (j + 1) * 0x9E3779B97F4A7C15ull;
        z ^= z >> 29;
        const uint64_t row = z % store_rows;
        copy_row<G>(reinterpret_cast<const v4u*>(store + row * row_bytes),
                    reinterpret_cast<v4u*>(out + j * (uint64_t)row_bytes), nullptr, row_u4, sub);
    }
}

// accum: 0 = no accumulator; otherwise bit 0 = this gather closes its group, bit 1 = it opened the group
__global__ void finalize_kernel(Ctl* ctl, StatsRec* rec, uint64_t seq, const uint32_t* n_u, int accum) {
    publish_stats(ctl, rec, seq, *n_u, accum);
}

inline int lanes_per_row(uint32_t row_bytes) {
    if (row_bytes >= 1024) return 64;
    if (row_bytes >= 512) return 32;
    if (row_bytes >= 256) return 16;
    return 8;
}

inline uint32_t row_grid(uint64_t rows, int g, int blocks) {
    const uint64_t per_block = MV_THREADS / g;
    uint64_t b = (rows + per_block - 1) / per_block;
    if (b < 1) b = 1;
    return (uint32_t)(b > (uint64_t)blocks ? (uint64_t)blocks : b);
}

#define GIDS_DISPATCH_G(g, CALL)      \
    switch (g) {                      \
        case 64: { constexpr int G = 64; CALL; } break; \
        case 32: { constexpr int G = 32; CALL; } break; \
        case 16: { constexpr int G = 16; CALL; } break; \
        default: { constexpr int G = 8; CALL; } break;  \
    }

}  // namespace

// chunks a link wave should expect at least (GIDS_LINK_SPREAD; 0: keep the largest chunk).  Eight: with two, the
// last chunks of a 24 k-row list (32 rows each, four per wave) end up to 0.2 ms apart and the link idles meanwhile
// (Skew 0.839 -> 0.858 of its roofline, Medium 0.844 -> 0.858, Large unchanged).
inline uint32_t link_spread_knob() {
    static const uint32_t link_spread = [] {
        const char* e = getenv("GIDS_LINK_SPREAD");
        const int v = e ? atoi(e) : 8;
        return (uint32_t)((v >= 0 && v <= 64) ? v : 8);
    }();
    return link_spread;
}

template <typename IdT>
void launch_move(const CacheView<IdT>& c, const IdT* unique, BatchHdr* hdr, uint64_t n_upper,
                 const uint64_t* plan, char* out, IdT* unique_out, int blocks, int link_blocks_max, hipStream_t s) {
    const int g = lanes_per_row(c.row_bytes);
    // a wave of the HBM half takes 16 plan entries per step, one of the link half 64
    static const uint32_t hbm_ch = [] {
        const char* e = getenv("GIDS_HBM_CHUNK");
        const int v = e ? atoi(e) : 16;
        return (uint32_t)((v == 1 || v == 2 || v == 4 || v == 8 || v == 16 || v == 32 || v == 64) ? v : 16);
    }();
    const uint32_t hbm_blocks = row_grid(n_upper, 64 / (int)hbm_ch, blocks);   // 4 waves x hbm_ch rows per workgroup step
    // the link half scans 64 entries per wave step when the list is long enough to keep all its waves busy
    // that way, fewer otherwise (short lists are latency-bound: spread them over more waves)
    static const uint32_t link_ch_max = [] {
        const char* e = getenv("GIDS_LINK_CHUNK");
        const int v = e ? atoi(e) : 64;
        return (uint32_t)((v == 4 || v == 8 || v == 16 || v == 32 || v == 64) ? v : 64);
    }();
    const uint32_t link_spread = link_spread_knob();
    uint32_t link_ch = link_ch_max;
    while (link_ch > 4 && n_upper / link_ch < (uint64_t)link_blocks_max * (MV_THREADS / 64)) link_ch >>= 1;
    const uint32_t link_blocks = row_grid(n_upper, 64 / (int)link_ch, link_blocks_max);
    GIDS_DISPATCH_G(g, hipLaunchKernelGGL((move_kernel<IdT, G>), dim3(link_blocks + hbm_blocks), dim3(MV_THREADS), 0,
                                          s, c, unique, hdr, plan, out, unique_out, link_blocks, link_ch, hbm_ch, link_spread));
}

template <typename IdT>
void launch_queue(const CacheView<IdT>& c, const AccumView& a, uint32_t group, const IdT* unique, const BatchHdr* hdr,
                  uint64_t n_upper, const uint64_t* plan, char* out, IdT* unique_out, hipStream_t s) {
    const uint32_t grid = row_grid(n_upper, 1, 1024);         // 4 waves x 64 entries per workgroup step
    hipLaunchKernelGGL(queue_kernel<IdT>, dim3(grid), dim3(MV_THREADS), 0, s, c, a, group, unique, hdr, plan, out,
                       unique_out);
}

template <typename IdT>
void launch_settle(const CacheView<IdT>& c, const AccumView& a, uint32_t group, int accum, const IdT* unique,
                   const uint32_t* n_u, uint64_t n_upper, const uint64_t* plan, BatchHdr* hdr, char* out,
                   IdT* unique_out, StatsRec* rec, uint64_t seq, hipStream_t s) {
    // few workgroups: each ends with an atomic on one counter
    const uint32_t grid = row_grid(n_upper, 1, 256);
    hipLaunchKernelGGL(settle_kernel<IdT>, dim3(grid), dim3(MV_THREADS), 0, s, c, a, group, accum, unique, n_u, plan,
                       hdr, out, unique_out, rec, seq);
}

template <typename IdT>
void launch_group_move(const CacheView<IdT>& c, const AccumView& a, uint32_t par, uint64_t rows_upper,
                       int hbm_blocks_max, int link_blocks_max, const UniqCopies& u, const IdT* stage, hipStream_t s) {
    const int g = lanes_per_row(c.row_bytes);
    if (rows_upper < 1) rows_upper = 1;
    uint32_t link_ch = 64;
    while (link_ch > 4 && rows_upper / link_ch < (uint64_t)link_blocks_max * (MV_THREADS / 64)) link_ch >>= 1;
    const uint32_t link_blocks = row_grid(rows_upper, 64 / (int)link_ch, link_blocks_max);
    const uint32_t hbm_blocks = row_grid(rows_upper, 4, hbm_blocks_max);   // 4 waves x 16 operations per workgroup step
    bool any = false;
    for (uint32_t i = 0; i < u.n; i++) any |= u.dst[i] != nullptr;
    const uint32_t uniq_blocks = any ? u.n : 0;
    GIDS_DISPATCH_G(g, hipLaunchKernelGGL((group_move_kernel<G>), dim3(link_blocks + hbm_blocks + uniq_blocks),
                                          dim3(MV_THREADS), 0, s, c.ctl, a.fills[par], a.rcopies[par], c.cache_data,
                                          c.line_bytes, c.row_bytes, par, link_blocks, hbm_blocks, link_ch,
                                          link_spread_knob(), u, reinterpret_cast<const uint32_t*>(stage),
                                          (uint32_t)(sizeof(IdT) / 4)));
    const uint32_t copy_blocks = row_grid(rows_upper, g, 256);
    GIDS_DISPATCH_G(g, hipLaunchKernelGGL((group_copy_kernel<G>), dim3(copy_blocks), dim3(MV_THREADS), 0, s, c.ctl,
                                          a.wcopies[par], c.row_bytes, par));
}

void launch_calibrate(const char* store, uint64_t store_rows, uint32_t row_bytes, char* out, uint32_t n,
                      hipStream_t s) {
    const int g = lanes_per_row(row_bytes);
    const uint32_t grid = row_grid(n, g, 48);                 // the row mover's default link half
    GIDS_DISPATCH_G(g, hipLaunchKernelGGL((calibrate_kernel<G>), dim3(grid), dim3(MV_THREADS), 0, s, store, store_rows,
                                          row_bytes, out, n));
}

void launch_finalize(Ctl* ctl, StatsRec* rec, uint64_t seq, const uint32_t* n_u, int accum, hipStream_t s) {
    hipLaunchKernelGGL(finalize_kernel, dim3(1), dim3(1), 0, s, ctl, rec, seq, n_u, accum);
}

#define GIDS_INSTANTIATE(IdT)                                                                                       \
    template void launch_move<IdT>(const CacheView<IdT>&, const IdT*, BatchHdr*, uint64_t, const uint64_t*,         \
                                   char*, IdT*, int, int, hipStream_t);                                             \
    template void launch_queue<IdT>(const CacheView<IdT>&, const AccumView&, uint32_t, const IdT*, const BatchHdr*, \
                                    uint64_t, const uint64_t*, char*, IdT*, hipStream_t);                           \
    template void launch_settle<IdT>(const CacheView<IdT>&, const AccumView&, uint32_t, int, const IdT*,            \
                                     const uint32_t*, uint64_t, const uint64_t*, BatchHdr*, char*, IdT*, StatsRec*, \
                                     uint64_t, hipStream_t);                                                        \
    template void launch_group_move<IdT>(const CacheView<IdT>&, const AccumView&, uint32_t, uint64_t, int, int,     \
                                         const UniqCopies&, const IdT*, hipStream_t);
GIDS_INSTANTIATE(int32_t)
GIDS_INSTANTIATE(int64_t)

}  // namespace gids
