"""A convenience wrapper for harnesses (tests, benchmark, smoke check): owns
the store / cache handles and the torch tensors whose device pointers go
through the C ABI.  It moves arguments only; it computes nothing."""
from __future__ import annotations

import ctypes as C

import numpy as np
import torch

from . import binding as B


class GatherSession:
    def __init__(self, n_rows: int, row_bytes: int, id_dtype, lines: int, ways: int, line_bytes: int,
                 window: int = 0, accum_threshold: int = 0, host_store: torch.Tensor | None = None,
                 store_handle: int | None = None):
        if not torch.cuda.is_available():
            raise RuntimeError("GatherSession needs a GPU: the gather has no CPU path")
        self.n_rows, self.row_bytes = n_rows, row_bytes
        self.id_dtype = np.dtype(id_dtype)
        self.torch_id = torch.int32 if self.id_dtype.itemsize == 4 else torch.int64
        self.window = window
        self._host_store = host_store
        self._owns_store = store_handle is None
        self.store = store_handle if store_handle is not None else B.gids_store_create(
            n_rows, row_bytes, self.id_dtype.itemsize, None if host_store is None else host_store.data_ptr())
        self.cache = None
        try:
            self.cache = B.gids_cache_create(self.store, lines, ways, line_bytes, window, accum_threshold)
        except Exception:
            if self._owns_store:
                B.gids_store_destroy(self.store)
            self.store = None
            raise
        self.lines = lines
        self._keep = []          # tensors the library may still read or write (outputs awaiting a flush)

    # -- the host table ----------------------------------------------------
    def store_view(self) -> np.ndarray:
        """The pinned host table as a uint8 array [n_rows, row_bytes] (to fill it)."""
        ptr = B.gids_store_host_ptr(self.store)
        buf = (C.c_uint8 * (self.n_rows * self.row_bytes)).from_address(ptr)
        return np.ctypeslib.as_array(buf).reshape(self.n_rows, self.row_bytes)

    def store_address(self) -> int:
        return B.gids_store_host_ptr(self.store)

    def pin_hot(self, ids) -> None:
        ids = np.ascontiguousarray(np.asarray(ids, dtype=self.id_dtype))
        B.gids_cpu_buffer_pin(self.cache, ids.ctypes.data, len(ids))

    def set_policy(self, policy: int, seed: int = 0) -> None:
        B.gids_cache_set_policy(self.cache, policy, seed)

    def set_accum_mode(self, mode: int) -> None:
        B.gids_cache_set_accum_mode(self.cache, mode)

    def set_group_dedup(self, on: bool) -> None:
        B.gids_cache_set_group_dedup(self.cache, on)

    def set_rows_per_line(self, rows: int) -> None:
        B.gids_cache_set_rows_per_line(self.cache, rows)

    def reserve(self, max_ids: int) -> None:
        B.gids_cache_reserve(self.cache, max_ids)

    # -- device-side calls -------------------------------------------------
    def to_device(self, raw) -> torch.Tensor:
        raw = np.ascontiguousarray(np.asarray(raw, dtype=self.id_dtype))
        return torch.from_numpy(raw).cuda() if len(raw) else torch.empty(0, dtype=self.torch_id, device="cuda")

    def push(self, ids_dev: torch.Tensor, stream: torch.cuda.Stream | None = None) -> None:
        stream = (stream or torch.cuda.current_stream()).cuda_stream
        B.gids_window_push(self.cache, ids_dev.data_ptr() if ids_dev.numel() else None, ids_dev.numel(), stream)
        self._keep.append(ids_dev)

    def push_dev(self, ids_dev: torch.Tensor, n_dev: torch.Tensor, stream: torch.cuda.Stream | None = None) -> None:
        """Push a list whose length lives in device memory (n_dev: uint32/int32 scalar tensor)."""
        stream = (stream or torch.cuda.current_stream()).cuda_stream
        B.gids_window_push_dev(self.cache, ids_dev.data_ptr(), ids_dev.numel(), n_dev.data_ptr(), stream)
        self._keep.append((ids_dev, n_dev))

    def gather(self, ids_dev: torch.Tensor | None, out: torch.Tensor, unique: torch.Tensor | None = None,
               inverse: torch.Tensor | None = None, stream: torch.cuda.Stream | None = None) -> int:
        """Enqueue one gather; returns its sequence number (for stats)."""
        stream = (stream or torch.cuda.current_stream()).cuda_stream
        seq = B.gids_cache_gathers(self.cache)
        n = 0 if ids_dev is None else ids_dev.numel()
        if n == 0:
            inverse = None
        B.gids_gather(self.cache, ids_dev.data_ptr() if n else None, n, out.data_ptr(), out.shape[0],
                      None if unique is None else unique.data_ptr(), None if inverse is None else inverse.data_ptr(),
                      stream)
        if len(self._keep) > 64:
            del self._keep[:-64]
        return seq

    def gather_many(self, pushes, outs, uniques=None, stream: torch.cuda.Stream | None = None,
                    push_stream: torch.cuda.Stream | None = None) -> int:
        """k merged steps: pushes[i] (a device ID tensor or None) is pushed, then the window's head is gathered
        into outs[i] (and uniques[i]).  Returns the sequence number of step 0."""
        stream = (stream or torch.cuda.current_stream()).cuda_stream
        push_stream = stream if push_stream is None else push_stream.cuda_stream
        seq = B.gids_cache_gathers(self.cache)
        any_push = any(p is not None for p in pushes)
        B.gids_gather_many(self.cache,
                           # (an empty list is still a push: any non-null address, it is never read)
                           [None if p is None else (p.data_ptr() or 8) for p in pushes] if any_push else None,
                           [0 if p is None else p.numel() for p in pushes],
                           [o.data_ptr() for o in outs], [o.shape[0] for o in outs],
                           None if uniques is None else [None if u is None else u.data_ptr() for u in uniques],
                           push_stream, stream)
        self._keep.extend(p for p in pushes if p is not None)
        if len(self._keep) > 96:
            del self._keep[:-96]
        return seq

    def flush(self) -> None:
        B.gids_flush(self.cache, torch.cuda.current_stream().cuda_stream)

    def stats(self, seq: int) -> B.gids_stats:
        return B.gids_stats_read(self.cache, seq)

    def snapshot(self):
        tags = np.empty(self.lines, dtype=np.int64)
        stamps = np.empty(self.lines, dtype=np.int64)
        B.gids_cache_snapshot(self.cache, tags.ctypes.data, stamps.ctypes.data)
        return tags, stamps

    def close(self) -> None:
        if self.cache:
            torch.cuda.synchronize()
            B.gids_cache_destroy(self.cache)
            self.cache = None
        if self.store:
            if self._owns_store:
                B.gids_store_destroy(self.store)
            self.store = None
        self._keep.clear()

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class GraphSampler:
    """Owns a gids_graph handle; argument marshalling for gids_sample."""

    def __init__(self, indptr: np.ndarray, indices: np.ndarray, zero_copy: bool = False):
        if not torch.cuda.is_available():
            raise RuntimeError("GraphSampler needs a GPU")
        self.id_dtype = indices.dtype
        self.torch_id = torch.int32 if indices.dtype.itemsize == 4 else torch.int64
        self.n_nodes = len(indptr) - 1
        if zero_copy:                      # the arrays must live in pinned (hipHostMalloc) memory
            self._indptr = torch.from_numpy(np.ascontiguousarray(indptr, dtype=np.int64)).pin_memory()
            self._indices = torch.from_numpy(np.ascontiguousarray(indices)).pin_memory()
            a, b = self._indptr.data_ptr(), self._indices.data_ptr()
        else:
            self._indptr = np.ascontiguousarray(indptr, dtype=np.int64)
            self._indices = np.ascontiguousarray(indices)
            a, b = self._indptr.ctypes.data, self._indices.ctypes.data
        self.graph = B.gids_graph_create(self.n_nodes, a, b, indices.dtype.itemsize, zero_copy)
        if not zero_copy:
            self._indptr = self._indices = None

    def capacity(self, fanouts, n_seeds: int) -> int:
        return B.gids_sample_capacity(fanouts, n_seeds)

    def sample(self, seed: int, batch: int, fanouts, n_seeds: int, raw: torch.Tensor, n_raw: torch.Tensor,
               stream: torch.cuda.Stream | None = None, rank_table: torch.Tensor | None = None, perm=(0, 0)) -> None:
        stream = (stream or torch.cuda.current_stream()).cuda_stream
        B.gids_sample(self.graph, seed, batch, fanouts, n_seeds, raw.data_ptr(), raw.numel(), n_raw.data_ptr(), stream,
                      None if rank_table is None else rank_table.data_ptr(), perm[0], perm[1])

    def visit_scores(self, fanouts, n_seeds: int) -> torch.Tensor:
        """Expected appearances per node and minibatch, 32.32 fixed point (int64 tensor on the device)."""
        scores = torch.empty(self.n_nodes, dtype=torch.int64, device="cuda")
        B.gids_graph_visit_scores(self.graph, fanouts, n_seeds, scores.data_ptr(),
                                  torch.cuda.current_stream().cuda_stream)
        return scores

    def reverse_pagerank(self, damping_q16: int = 55705, n_iters: int = 20) -> torch.Tensor:
        """Weighted reverse PageRank per node, total mass 2^44 (int64 tensor on the device)."""
        scores = torch.empty(self.n_nodes, dtype=torch.int64, device="cuda")
        B.gids_graph_reverse_pagerank(self.graph, damping_q16, n_iters, scores.data_ptr(),
                                      torch.cuda.current_stream().cuda_stream)
        return scores

    def close(self) -> None:
        if self.graph:
            torch.cuda.synchronize()
            B.gids_graph_destroy(self.graph)
            self.graph = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
