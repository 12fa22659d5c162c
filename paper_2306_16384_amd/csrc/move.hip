// Row movement of the feature gather (GIDS paper, Section 2.2.3 for the
// gather, Section 3.2 for batching accesses across minibatches, Section 3.3
// for rows redirected to the CPU buffer).
//
//   move      one group of lanes per output row, 16 bytes per lane per access:
//             a hit copies cache line -> output (HBM -> HBM); a CPU-buffer hit
//             copies pinned host row -> output; a miss reads the host store row
//             once and writes it to the output and, when a victim line was
//             found, to that line (the "line fill"), then publishes the line's
//             tag and stamp.
//   queue     the accumulator's variant: rows that cross the host link are not
//             moved but appended to a fill queue; a hit on a line whose fill is
//             still queued becomes a queued copy from the output row that fill
//             will write.  Hits on lines that hold data are copied at once.
//   flush     moves every queued fill, then every queued copy, once enough are
//             pending (or on request).
//   finalize  publishes the minibatch's counters to host-visible memory and
//             advances the minibatch stamp.
#include "gids_dev.h"

namespace gids {

namespace {

constexpr int MV_THREADS = 256;
constexpr int MV_UNROLL = 4;

template <int G>
__device__ __forceinline__ void copy_row(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                         uint4* __restrict__ dst2, uint32_t row_u4, uint32_t sub) {
    for (uint32_t k0 = 0; k0 < row_u4; k0 += G * MV_UNROLL) {
        uint4 buf[MV_UNROLL];
#pragma unroll
        for (int u = 0; u < MV_UNROLL; u++) {
            const uint32_t k = k0 + u * G + sub;
            if (k < row_u4) buf[u] = src[k];
        }
#pragma unroll
        for (int u = 0; u < MV_UNROLL; u++) {
            const uint32_t k = k0 + u * G + sub;
            if (k < row_u4) {
                dst[k] = buf[u];
                if (dst2) dst2[k] = buf[u];
            }
        }
    }
}

template <typename IdT>
__device__ __forceinline__ void clear_miss_bit_word(const CacheView<IdT>& c, uint64_t v) {
    uint64_t set, round;
    if (c.use32) {
        const uint32_t q = (uint32_t)v / (uint32_t)c.n_sets;
        round = q;
        set = (uint32_t)v - q * (uint32_t)c.n_sets;
    } else {
        round = v / c.n_sets;
        set = v - round * c.n_sets;
    }
    c.missmask[set * c.words_per_set + (round >> 6)] = 0ull;
}

// The first `link_blocks` workgroups move the rows that cross the host link
// (CPU-buffer rows, store rows), the others the rows that stay in HBM (hits).
// The link is saturated by a few hundred workgroups and loses a few percent
// with thousands, while HBM needs thousands; both halves run concurrently.
template <typename IdT, int G>
__global__ __launch_bounds__(MV_THREADS) void move_kernel(CacheView<IdT> c, const IdT* __restrict__ unique,
                                                          const uint32_t* __restrict__ n_u_ptr,
                                                          const uint64_t* __restrict__ plan, char* __restrict__ out,
                                                          uint32_t link_blocks) {
    const Ctl* ctl = c.ctl;
    if (ctl->error) return;
    const uint32_t n_u = *n_u_ptr;
    const uint32_t row_u4 = c.row_bytes >> 4;
    const uint32_t sub = threadIdx.x % G;
    const int32_t stamp = (int32_t)ctl->stamp;
    const bool link_role = blockIdx.x < link_blocks;
    const uint32_t role_block = link_role ? blockIdx.x : blockIdx.x - link_blocks;
    const uint32_t role_blocks = link_role ? link_blocks : gridDim.x - link_blocks;
    const uint64_t g0 = ((uint64_t)role_block * MV_THREADS + threadIdx.x) / G;
    const uint64_t n_groups = (uint64_t)role_blocks * MV_THREADS / G;
    for (uint64_t j = g0; j < n_u; j += n_groups) {
        const uint64_t e = plan[j];
        const uint64_t kind = e >> PLAN_SHIFT, idx = e & PLAN_INDEX_MASK;
        if ((kind != PLAN_HIT) != link_role) continue;
        const uint64_t v = (uint64_t)unique[j];
        const char* src;
        char* line = nullptr;
        if (kind == PLAN_HIT) src = c.cache_data + idx * c.line_bytes;
        else if (kind == PLAN_CPU) src = c.cpubuf + idx * c.row_bytes;
        else {
            src = c.store + v * c.row_bytes;
            if (kind == PLAN_INSTALL) line = c.cache_data + idx * c.line_bytes;
        }
        copy_row<G>(reinterpret_cast<const uint4*>(src), reinterpret_cast<uint4*>(out + j * c.row_bytes),
                    reinterpret_cast<uint4*>(line), row_u4, sub);
        if (sub == 0 && kind >= PLAN_INSTALL) {
            if (kind == PLAN_INSTALL) {
                c.tags[idx] = (IdT)v;
                c.stamps[idx] = stamp;
            }
            clear_miss_bit_word(c, v);
        }
    }
}

template <typename IdT, int G>
__global__ __launch_bounds__(MV_THREADS) void queue_kernel(CacheView<IdT> c, const IdT* __restrict__ unique,
                                                           const uint32_t* __restrict__ n_u_ptr,
                                                           const uint64_t* __restrict__ plan, char* __restrict__ out,
                                                           FillOp* __restrict__ fills, CopyOp* __restrict__ copies) {
    Ctl* ctl = c.ctl;
    if (ctl->error) return;
    const uint32_t n_u = *n_u_ptr;
    const uint32_t row_u4 = c.row_bytes >> 4;
    const uint32_t sub = threadIdx.x % G;
    const int32_t stamp = (int32_t)ctl->stamp;
    const uint64_t g0 = ((uint64_t)blockIdx.x * MV_THREADS + threadIdx.x) / G;
    const uint64_t n_groups = (uint64_t)gridDim.x * MV_THREADS / G;
    for (uint64_t j = g0; j < n_u; j += n_groups) {
        const uint64_t e = plan[j];
        const uint64_t kind = e >> PLAN_SHIFT, idx = e & PLAN_INDEX_MASK;
        const uint64_t v = (uint64_t)unique[j];
        char* dst = out + j * c.row_bytes;
        if (kind == PLAN_HIT) {
            const uint32_t p = c.pending[idx];             // written only by earlier gathers or flushes
            if (p == NO_OP) {
                copy_row<G>(reinterpret_cast<const uint4*>(c.cache_data + idx * c.line_bytes),
                            reinterpret_cast<uint4*>(dst), nullptr, row_u4, sub);
            } else if (sub == 0) {                         // the line's bytes are still on their way
                const uint32_t q = atomicAdd(&ctl->pend_copy, 1u);
                copies[q].src = fills[p].dst_out;
                copies[q].dst_out = dst;
                atomicAdd(&ctl->deferred, 1u);
            }
            continue;
        }
        if (sub != 0) continue;
        const uint32_t q = atomicAdd(&ctl->pend_fill, 1u);
        atomicAdd(&ctl->deferred, 1u);
        fills[q].dst_out = dst;
        fills[q].dst_line = NO_LINE;
        if (kind == PLAN_CPU) {
            fills[q].src = c.cpubuf + idx * c.row_bytes;
            continue;
        }
        fills[q].src = c.store + v * c.row_bytes;
        if (kind == PLAN_INSTALL) {
            const uint32_t old = c.pending[idx];
            if (old != NO_OP) fills[old].dst_line = NO_LINE;   // superseded before it ever ran: output only
            fills[q].dst_line = idx;
            c.pending[idx] = q;
            c.tags[idx] = (IdT)v;
            c.stamps[idx] = stamp;
        }
        clear_miss_bit_word(c, v);
    }
}

__device__ __forceinline__ bool flush_now(const Ctl* ctl, uint64_t threshold, int force) {
    return force || ((uint64_t)ctl->pend_fill + ctl->pend_copy >= threshold);
}

template <typename IdT, int G>
__global__ __launch_bounds__(MV_THREADS) void flush_fill_kernel(CacheView<IdT> c, const FillOp* __restrict__ fills,
                                                                uint64_t threshold, int force) {
    const Ctl* ctl = c.ctl;
    if (ctl->error || !flush_now(ctl, threshold, force)) return;
    const uint32_t n = ctl->pend_fill;
    const uint32_t row_u4 = c.row_bytes >> 4;
    const uint32_t sub = threadIdx.x % G;
    const uint64_t g0 = ((uint64_t)blockIdx.x * MV_THREADS + threadIdx.x) / G;
    const uint64_t n_groups = (uint64_t)gridDim.x * MV_THREADS / G;
    for (uint64_t i = g0; i < n; i += n_groups) {
        const FillOp op = fills[i];
        char* line = op.dst_line == NO_LINE ? nullptr : c.cache_data + op.dst_line * c.line_bytes;
        copy_row<G>(reinterpret_cast<const uint4*>(op.src), reinterpret_cast<uint4*>(op.dst_out),
                    reinterpret_cast<uint4*>(line), row_u4, sub);
        if (sub == 0 && line) c.pending[op.dst_line] = NO_OP;
    }
}

template <typename IdT, int G>
__global__ __launch_bounds__(MV_THREADS) void flush_copy_kernel(CacheView<IdT> c, const CopyOp* __restrict__ copies,
                                                                uint64_t threshold, int force) {
    const Ctl* ctl = c.ctl;
    if (ctl->error || !flush_now(ctl, threshold, force)) return;
    const uint32_t n = ctl->pend_copy;
    const uint32_t row_u4 = c.row_bytes >> 4;
    const uint32_t sub = threadIdx.x % G;
    const uint64_t g0 = ((uint64_t)blockIdx.x * MV_THREADS + threadIdx.x) / G;
    const uint64_t n_groups = (uint64_t)gridDim.x * MV_THREADS / G;
    for (uint64_t i = g0; i < n; i += n_groups) {
        const CopyOp op = copies[i];
        copy_row<G>(reinterpret_cast<const uint4*>(op.src), reinterpret_cast<uint4*>(op.dst_out), nullptr, row_u4,
                    sub);
    }
}

// after the flush kernels: empty the queues if they ran
__global__ void flush_done_kernel(Ctl* ctl, uint64_t threshold, int force) {
    if (ctl->error) return;
    if (flush_now(ctl, threshold, force)) {
        ctl->pend_fill = 0;
        ctl->pend_copy = 0;
        ctl->deferred = 0;
    }
}

__global__ void finalize_kernel(Ctl* ctl, StatsRec* rec, uint64_t seq, const uint32_t* n_u) {
    const uint32_t err = ctl->error;
    rec->n_unique = err ? 0 : *n_u;
    rec->n_hit = ctl->cnt_hit;
    rec->n_cpu_hit = ctl->cnt_cpu;
    rec->n_miss = ctl->cnt_miss;
    rec->n_bypass = ctl->cnt_bypass;
    rec->n_pending = (uint64_t)ctl->pend_fill + ctl->pend_copy;
    rec->flushed = ctl->deferred == 0;
    rec->status = -(int32_t)err;
    __threadfence_system();
    rec->seq = seq;                       // written last: a record whose seq matches is complete
    __threadfence_system();
    if (!err) ctl->stamp += 1;
    ctl->cnt_hit = ctl->cnt_cpu = ctl->cnt_miss = ctl->cnt_bypass = 0;
    ctl->deferred = 0;
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

template <typename IdT>
void launch_move(const CacheView<IdT>& c, const IdT* unique, const uint32_t* n_u, uint64_t n_upper,
                 const uint64_t* plan, char* out, int blocks, int link_blocks_max, hipStream_t s) {
    const int g = lanes_per_row(c.row_bytes);
    const uint32_t hbm_blocks = row_grid(n_upper, g, blocks);
    const uint32_t link_blocks = row_grid(n_upper, g, link_blocks_max);
    GIDS_DISPATCH_G(g, hipLaunchKernelGGL((move_kernel<IdT, G>), dim3(link_blocks + hbm_blocks), dim3(MV_THREADS), 0,
                                          s, c, unique, n_u, plan, out, link_blocks));
}

template <typename IdT>
void launch_queue(const CacheView<IdT>& c, const IdT* unique, const uint32_t* n_u, uint64_t n_upper,
                  const uint64_t* plan, char* out, FillOp* fills, CopyOp* copies, uint32_t, int blocks,
                  hipStream_t s) {
    const int g = lanes_per_row(c.row_bytes);
    const uint32_t grid = row_grid(n_upper, g, blocks);
    GIDS_DISPATCH_G(g, hipLaunchKernelGGL((queue_kernel<IdT, G>), dim3(grid), dim3(MV_THREADS), 0, s, c, unique,
                                          n_u, plan, out, fills, copies));
}

template <typename IdT>
void launch_flush(const CacheView<IdT>& c, FillOp* fills, CopyOp* copies, uint64_t threshold, bool force,
                  int blocks, hipStream_t s) {
    const int g = lanes_per_row(c.row_bytes);
    const int f = force ? 1 : 0;
    GIDS_DISPATCH_G(g, hipLaunchKernelGGL((flush_fill_kernel<IdT, G>), dim3(blocks), dim3(MV_THREADS), 0, s, c,
                                          fills, threshold, f));
    GIDS_DISPATCH_G(g, hipLaunchKernelGGL((flush_copy_kernel<IdT, G>), dim3(blocks), dim3(MV_THREADS), 0, s, c,
                                          copies, threshold, f));
    hipLaunchKernelGGL(flush_done_kernel, dim3(1), dim3(1), 0, s, c.ctl, threshold, f);
}

void launch_finalize(Ctl* ctl, StatsRec* rec, uint64_t seq, const uint32_t* n_u, hipStream_t s) {
    hipLaunchKernelGGL(finalize_kernel, dim3(1), dim3(1), 0, s, ctl, rec, seq, n_u);
}

#define GIDS_INSTANTIATE(IdT)                                                                                       \
    template void launch_move<IdT>(const CacheView<IdT>&, const IdT*, const uint32_t*, uint64_t, const uint64_t*,   \
                                   char*, int, int, hipStream_t);                                                        \
    template void launch_queue<IdT>(const CacheView<IdT>&, const IdT*, const uint32_t*, uint64_t, const uint64_t*,  \
                                    char*, FillOp*, CopyOp*, uint32_t, int, hipStream_t);                           \
    template void launch_flush<IdT>(const CacheView<IdT>&, FillOp*, CopyOp*, uint64_t, bool, int, hipStream_t);
GIDS_INSTANTIATE(int32_t)
GIDS_INSTANTIATE(int64_t)

}  // namespace gids
