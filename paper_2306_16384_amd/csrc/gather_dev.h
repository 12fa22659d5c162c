// Device code shared by the per-step kernels and the fused classification
// kernel: appending one plan entry to the accumulator's lists, and publishing
// a minibatch's counters.
#pragma once

#include "gids_dev.h"

namespace gids {

// Where queue_entry keeps what it knows of a cache line between the minibatches of a group: the group in which
// the line's fill was queued and that fill's index, the group in which a copy out of the line was last queued.
// The per-step kernels keep these words in device memory, indexed by line.
struct LineWordsGlobal {
    static constexpr bool deferred = false;                   // a line's fill is queued when the line is installed
    uint32_t* pending;
    uint32_t* fillgrp;
    uint32_t* hitgrp;
    const FillOp* fills;
    __device__ __forceinline__ uint32_t fill_group(uint64_t line, uint32_t) const { return fillgrp[line]; }
    __device__ __forceinline__ uint32_t hit_group(uint64_t line, uint32_t) const { return hitgrp[line]; }
    __device__ __forceinline__ uint32_t pending_fill(uint64_t line, uint32_t) const { return pending[line]; }
    // the output row the line's queued fill writes
    __device__ __forceinline__ void* pending_out(uint64_t, uint32_t, uint32_t pd) const { return fills[pd].dst_out; }
    __device__ __forceinline__ void note_fill(uint64_t line, uint32_t, uint32_t group, uint32_t q, char*) const {
        fillgrp[line] = group;
        pending[line] = q;
    }
    __device__ __forceinline__ void note_hit(uint64_t line, uint32_t, uint32_t group) const { hitgrp[line] = group; }
};

// Where queue_entry takes places in the group's three lists (0 fills, 1 rcopies, 2 wcopies) from: the lists'
// counters in device memory, one atomic per wavefront and list.
struct PlacesGlobal {
    Ctl* ctl;
    uint32_t par;
    __device__ __forceinline__ uint32_t take(int list, uint32_t n) const {
        return atomicAdd(list == 0 ? &ctl->q_fill[par] : list == 1 ? &ctl->q_rcopy[par] : &ctl->q_wcopy[par], n);
    }
};

// The accumulator's treatment of plan entry j (Section 3.2: nothing moves while a group of minibatches is
// open; every row becomes an operation in the group's lists).  Called by all 64 lanes of a wavefront
// together, `valid` false for lanes without an entry; the lanes' entries may be any distinct j.
//   fills    rows that cross the host link (CPU-buffer rows, store rows), each to its output row and, for an
//            installed miss, to its cache line;
//   rcopies  hits on lines that hold their bytes: cache line -> output row;
//   wcopies  copies that must run after the fills: a hit on a line whose fill is queued in the same group
//            reads the output row that fill writes; an installed miss whose line a queued rcopy still reads
//            (the line was hit earlier in the group and evicted since) fills its line late, from its own
//            output row, so that the rcopy sees the old bytes.
// A line installed twice in one group is filled by the last install only (the earlier fill keeps its output
// row).  Every line is touched by at most one plan entry per minibatch, so the per-line words are written
// without atomics.  `lw` holds the per-line words, `local` is the line's index there where that is not the
// line number; `places` hands out list positions.
// With LineWords::deferred the fill of an installed line is not queued here: it waits in the line's words (node,
// output row, whether it is late) until the line is installed again in the same group (then it goes out for its
// output row only) or until the holder of the words queues what is left when the group ends; no queued operation
// is ever read or changed again.
// `first_out` (per lane, or nullptr): for a CPU-buffer row, the word that remembers which output row the group's
// first fill of that row writes (nullptr: none yet).  A later minibatch of the group that needs the same row
// copies it from there, after the fills, instead of reading it over the link again.
// Returns whether this lane's entry was such a copy.
template <typename IdT, typename LineWords, typename Places>
__device__ __forceinline__ bool queue_entry(const CacheView<IdT>& c, const AccumView& a, const LineWords& lw,
                                            const Places& places, uint32_t group, bool valid, uint64_t j, uint64_t e,
                                            uint64_t v, uint32_t local, char* __restrict__ out,
                                            IdT* __restrict__ unique_out, char** first_out = nullptr) {
    Ctl* ctl = c.ctl;
    const uint32_t par = group & 1u;
    FillOp* __restrict__ fills = a.fills[par];
    CopyOp* __restrict__ rcopies = a.rcopies[par];
    CopyOp* __restrict__ wcopies = a.wcopies[par];
    const uint32_t lane = threadIdx.x & 63;
    const uint64_t kind = valid ? e >> PLAN_SHIFT : PLAN_HIT, idx = e & PLAN_INDEX_MASK;
    if (valid && unique_out) unique_out[j] = (IdT)v;
    const bool has_line = valid && (kind == PLAN_HIT || kind == PLAN_INSTALL);
    uint32_t fg = ~0u, hg = ~0u, pd = NO_OP;
    if (has_line) {
        fg = lw.fill_group(idx, local);
        hg = lw.hit_group(idx, local);
        pd = lw.pending_fill(idx, local);
    }
    const bool open_fill = has_line && fg == group;               // the line's fill is queued in this group
    const bool is_wait = valid && kind == PLAN_HIT && open_fill;
    const bool is_ready = valid && kind == PLAN_HIT && !open_fill;
    const bool is_late = valid && kind == PLAN_INSTALL && hg == group;   // a queued rcopy still reads the old bytes
    // a fill now: every row that crosses the link; deferred, an installed line's own fill waits and only the one
    // it supersedes goes out
    char* again_from = nullptr;                                   // the output row that already receives this CPU-buffer row
    if (valid && kind == PLAN_CPU && first_out) again_from = *first_out;
    const bool is_again = again_from != nullptr;
    const bool is_fill = valid && kind != PLAN_HIT && !is_again &&
                         !(LineWords::deferred && kind == PLAN_INSTALL && !open_fill);
    const uint64_t fb = __ballot(is_fill), rb = __ballot(is_ready),
                   wb = __ballot(is_wait || is_again || (is_late && !LineWords::deferred));
    uint32_t fbase = 0, rbase = 0, wbase = 0;
    if (lane == 0) {
        if (fb) fbase = places.take(0, (uint32_t)__popcll(fb));
        if (rb) rbase = places.take(1, (uint32_t)__popcll(rb));
        if (wb) wbase = places.take(2, (uint32_t)__popcll(wb));
    }
    fbase = __shfl(fbase, 0);
    rbase = __shfl(rbase, 0);
    wbase = __shfl(wbase, 0);
    // the host sizes the lists for the group's longest possible content; a list that would overflow all
    // the same is an error, never a write past its end
    if ((uint64_t)fbase + __popcll(fb) > a.cap || (uint64_t)rbase + __popcll(rb) > a.cap ||
        (uint64_t)wbase + __popcll(wb) > a.cap) {
        if (lane == 0) atomicCAS(&ctl->error, 0u, 7u /* -GIDS_E_SPACE */);
        return false;
    }
    const uint64_t below = (1ull << lane) - 1;
    char* dst = out + j * c.row_bytes;
    const uint32_t w = wbase + (uint32_t)__popcll(wb & below);
    if (is_fill) {
        const uint32_t q = fbase + (uint32_t)__popcll(fb & below);
        FillOp op;
        op.src = kind == PLAN_CPU ? c.cpubuf + idx * c.row_bytes : c.store + v * c.row_bytes;
        op.dst_out = dst;
        op.dst_line = NO_LINE;
        op.late = NO_OP;
        op.pad = 0;
        if constexpr (LineWords::deferred) {
            if (kind == PLAN_INSTALL) {                       // the fill that waited here: its output row only
                op.src = c.store + (uint64_t)lw.waiting_node(local) * c.row_bytes;
                op.dst_out = lw.pending_out(idx, local, pd);
            }
        } else if (kind == PLAN_INSTALL) {
            if (open_fill) {                                  // superseded before it ever ran: output only
                fills[pd].dst_line = NO_LINE;
                const uint32_t lt = fills[pd].late;
                if (lt != NO_OP) wcopies[lt].dst = nullptr;
            }
            char* line = c.cache_data + idx * c.line_bytes;
            if (is_late) {
                wcopies[w].src = dst;
                wcopies[w].dst = line;
                op.late = w;
            } else {
                op.dst_line = idx;
            }
            lw.note_fill(idx, local, group, q, dst);
        }
        fills[q] = op;
    }
    if constexpr (LineWords::deferred) {
        if (valid && kind == PLAN_INSTALL) lw.wait_fill(local, group, (uint32_t)v, is_late, dst);
    }
    if (is_wait) {
        wcopies[w].src = lw.pending_out(idx, local, pd);
        wcopies[w].dst = dst;
    }
    if (is_again) {
        wcopies[w].src = again_from;
        wcopies[w].dst = dst;
    } else if (valid && kind == PLAN_CPU && first_out) {
        *first_out = dst;
    }
    if (is_ready) {
        const uint32_t r = rbase + (uint32_t)__popcll(rb & below);
        rcopies[r].src = c.cache_data + idx * c.line_bytes;
        rcopies[r].dst = dst;
        lw.note_hit(idx, local, group);
    }
    return is_again;
}

// The same with everything in device memory, as the per-step kernels use it.  once_per_group: a CPU-buffer row
// that an earlier minibatch of the open group already fetches comes as a copy (CacheView::cpu_first, which the
// host clears when the group closes); the wavefront's count of such rows goes to Ctl::cnt_again.
template <typename IdT>
__device__ __forceinline__ void queue_entry(const CacheView<IdT>& c, const AccumView& a, uint32_t group, bool valid,
                                            uint64_t j, uint64_t e, uint64_t v, char* __restrict__ out,
                                            IdT* __restrict__ unique_out, bool once_per_group = false) {
    const LineWordsGlobal lw{c.pending, c.fillgrp, c.hitgrp, a.fills[group & 1u]};
    const PlacesGlobal places{c.ctl, group & 1u};
    char** first = nullptr;
    if (once_per_group && c.cpu_first && valid && (e >> PLAN_SHIFT) == PLAN_CPU) first = c.cpu_first + (e & PLAN_INDEX_MASK);
    const bool again = queue_entry(c, a, lw, places, group, valid, j, e, v, 0u, out, unique_out, first);
    if (once_per_group && c.cpu_first) {
        const uint64_t b = __ballot(again);
        if (b && (threadIdx.x & 63) == 0) atomicAdd(&c.ctl->cnt_again, (uint32_t)__popcll(b));
    }
}

__device__ __forceinline__ uint32_t ld_agent(const uint32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The counters of one gather go to its record in host-visible memory, the minibatch index advances.
// accum: 0 = no accumulator; otherwise bit 0 = this gather closes its group, bit 1 = it opened the group, bit 3
// = the group's parity, bits 8.. = the gather's position in its group.  One thread, after every other write of
// the gather.
__device__ __forceinline__ void publish_stats(Ctl* ctl, StatsRec* rec, uint64_t seq, uint32_t n_u, int accum) {
    const uint32_t err = ld_agent(&ctl->error);          // (another workgroup of the same launch may have set it)
    const uint32_t n = err ? 0 : n_u;
    rec->n_unique = n;
    rec->n_hit = ctl->cnt_hit;
    rec->n_cpu_hit = ctl->cnt_cpu;
    rec->n_miss = ctl->cnt_miss;
    rec->n_bypass = ctl->cnt_bypass;
    rec->n_line_fills = ctl->cnt_fill;
    rec->n_cpu_again = ctl->cnt_again;
    uint32_t queued = 0;
    int flushed = 1;
    if (accum) {                          // rows of the open group that have not moved when this gather ends
        const bool closes = (accum & 1) != 0, opens = (accum & 2) != 0;
        queued = closes ? 0u : (opens ? 0u : ctl->q_rows) + n;
        ctl->q_rows = queued;
        ctl->grp_nu[(accum >> 3) & 1][(accum >> 8) % MANY_MAX] = n;   // for the copy of its distinct-ID list
        flushed = closes ? 1 : 0;
    }
    rec->n_pending = queued;
    rec->flushed = flushed;
    rec->status = -(int32_t)err;
    __threadfence_system();
    rec->seq = seq;                       // written last: a record whose seq matches is complete
    __threadfence_system();
    if (!err) ctl->stamp += 1;
    ctl->cnt_hit = ctl->cnt_cpu = ctl->cnt_miss = ctl->cnt_bypass = ctl->cnt_fill = ctl->cnt_again = 0;
}

}  // namespace gids
