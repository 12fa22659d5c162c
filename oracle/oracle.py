"""ctypes front end of the CPU oracle (gids_oracle.c).

Test infrastructure only: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  Never by the HIP library or its binding.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gids_oracle.c")
_LIB = os.path.join(_HERE, "libgids_oracle.so")

OK, E_INVAL, E_NOMEM, E_RANGE, E_ORDER, E_FULL = 0, -1, -2, -3, -4, -5
CLS_HIT, CLS_CPU, CLS_MISS, CLS_BYPASS = 0, 1, 2, 3


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-Wall", "-Wextra", "-shared",
                               "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None
_i64p = np.ctypeslib.ndpointer(dtype=np.int64, flags="C_CONTIGUOUS")


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.go_mix64.restype = C.c_uint64
        L.go_mix64.argtypes = [C.c_uint64]
        L.go_graph_create.restype = C.c_void_p
        L.go_graph_create.argtypes = [C.c_uint64, C.c_int64, C.c_double, C.c_int, C.c_int64]
        L.go_graph_from_csr.restype = C.c_void_p
        L.go_graph_from_csr.argtypes = [C.c_int64, _i64p, _i64p]
        L.go_graph_free.argtypes = [C.c_void_p]
        L.go_graph_edges.restype = C.c_int64
        L.go_graph_edges.argtypes = [C.c_void_p]
        L.go_graph_indptr.restype = C.POINTER(C.c_int64)
        L.go_graph_indptr.argtypes = [C.c_void_p]
        L.go_graph_indices.restype = C.POINTER(C.c_int64)
        L.go_graph_indices.argtypes = [C.c_void_p]
        L.go_hot_nodes.argtypes = [C.c_void_p, C.c_int64, _i64p]
        L.go_sort_unique.restype = C.c_int64
        L.go_sort_unique.argtypes = [_i64p, C.c_int64, _i64p]
        L.go_sample.restype = C.c_int64
        L.go_sample.argtypes = [C.c_void_p, C.c_uint64, C.c_int64, np.ctypeslib.ndpointer(dtype=np.int32),
                                C.c_int, C.c_int64, _i64p, C.c_int64]
        L.go_sample_skewed.restype = C.c_int64
        L.go_sample_skewed.argtypes = [C.c_void_p, C.c_uint64, C.c_int64, np.ctypeslib.ndpointer(dtype=np.int32),
                                       C.c_int, C.c_int64, np.ctypeslib.ndpointer(dtype=np.uint64), C.c_int64,
                                       C.c_int64, _i64p, C.c_int64]
        L.go_visit_scores.argtypes = [C.c_void_p, np.ctypeslib.ndpointer(dtype=np.int32), C.c_int, C.c_int64,
                                      np.ctypeslib.ndpointer(dtype=np.uint64)]
        L.go_reverse_pagerank.argtypes = [C.c_void_p, C.c_uint32, C.c_int, np.ctypeslib.ndpointer(dtype=np.uint64)]
        L.go_feat_row.argtypes = [C.c_uint64, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.go_accum_threshold.restype = C.c_double
        L.go_accum_threshold.argtypes = [C.c_double, C.c_double, C.c_double, C.c_double, C.c_int]
        L.go_sim_create.restype = C.c_void_p
        L.go_sim_create.argtypes = [C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_void_p]
        L.go_sim_free.argtypes = [C.c_void_p]
        L.go_sim_set_hot.argtypes = [C.c_void_p, _i64p, C.c_int64]
        L.go_sim_set_policy.argtypes = [C.c_void_p, C.c_int32, C.c_uint64]
        L.go_sim_set_rows_per_line.argtypes = [C.c_void_p, C.c_int64]
        L.go_sim_set_accum.argtypes = [C.c_void_p, C.c_int64, C.c_int32]
        L.go_sim_flush.restype = C.c_int64
        L.go_sim_flush.argtypes = [C.c_void_p]
        L.go_sim_accum_last.argtypes = [C.c_void_p, _i64p]
        L.go_sim_push.argtypes = [C.c_void_p, _i64p, C.c_int64]
        L.go_sim_gather.restype = C.c_int64
        L.go_sim_gather.argtypes = [C.c_void_p, _i64p, C.c_int64, _i64p, C.c_void_p, _i64p, C.c_void_p]
        L.go_sim_tags.restype = C.POINTER(C.c_int64)
        L.go_sim_tags.argtypes = [C.c_void_p]
        L.go_sim_stamps.restype = C.POINTER(C.c_int64)
        L.go_sim_stamps.argtypes = [C.c_void_p]
        L.go_sim_reuse.restype = C.POINTER(C.c_int32)
        L.go_sim_reuse.argtypes = [C.c_void_p]
        L.go_sim_batch.restype = C.c_int64
        L.go_sim_batch.argtypes = [C.c_void_p]
        L.go_sim_window_count.restype = C.c_int32
        L.go_sim_window_count.argtypes = [C.c_void_p]
        _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__(f"oracle error {code}")
        self.code = code


def mix64(z: int) -> int:
    return int(lib().go_mix64(z & 0xFFFFFFFFFFFFFFFF))


def _ids(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int64))


class Graph:
    """The oracle's own seeded power-law graph (CSR, int64)."""

    def __init__(self, seed: int, n: int, ell: float = 1.0, p4: int = 4, d_max: int = 1, csr=None):
        if csr is None:
            self._h = lib().go_graph_create(seed, n, ell, p4, d_max)
        else:
            self._h = lib().go_graph_from_csr(n, _ids(csr[0]), _ids(csr[1]))
        if not self._h:
            raise OracleError(E_INVAL)
        self.n, self.seed = n, seed
        self.n_edges = int(lib().go_graph_edges(self._h))
        self.indptr = np.ctypeslib.as_array(lib().go_graph_indptr(self._h), shape=(n + 1,))
        self.indices = np.ctypeslib.as_array(lib().go_graph_indices(self._h), shape=(self.n_edges,))

    def hot_nodes(self, k: int) -> np.ndarray:
        out = np.empty(k, dtype=np.int64)
        rc = lib().go_hot_nodes(self._h, k, out)
        if rc:
            raise OracleError(rc)
        return out

    def visit_scores(self, fanouts, n_seeds: int) -> np.ndarray:
        """Expected appearances per node in a minibatch's raw list, 32.32 fixed point (uint64)."""
        out = np.zeros(self.n, dtype=np.uint64)
        rc = lib().go_visit_scores(self._h, np.asarray(fanouts, dtype=np.int32), len(fanouts), n_seeds, out)
        if rc:
            raise OracleError(rc)
        return out

    def reverse_pagerank(self, damping_q16: int, n_iters: int) -> np.ndarray:
        """Weighted reverse PageRank after n_iters power iterations, total mass 2^44 (uint64)."""
        out = np.zeros(self.n, dtype=np.uint64)
        rc = lib().go_reverse_pagerank(self._h, damping_q16, n_iters, out)
        if rc:
            raise OracleError(rc)
        return out

    def sample(self, seed: int, batch: int, fanouts, n_seeds: int, cap: int | None = None,
               rank_table: np.ndarray | None = None, perm=None) -> np.ndarray:
        """rank_table / perm = (mult, add): seed nodes Zipf-ranked through an affine permutation"""
        if cap is None:
            cap, w = n_seeds, n_seeds
            for f in fanouts:
                w *= f
                cap += w
        out = np.empty(max(cap, 1), dtype=np.int64)
        f32 = np.asarray(fanouts, dtype=np.int32)
        if rank_table is None:
            n = lib().go_sample(self._h, seed, batch, f32, len(fanouts), n_seeds, out, cap)
        else:
            n = lib().go_sample_skewed(self._h, seed, batch, f32, len(fanouts), n_seeds,
                                       np.ascontiguousarray(rank_table, dtype=np.uint64), perm[0], perm[1], out, cap)
        if n < 0:
            raise OracleError(int(n))
        return out[:n].copy()

    def __del__(self):
        if getattr(self, "_h", None):
            lib().go_graph_free(self._h)
            self._h = None


def sort_unique(raw) -> np.ndarray:
    raw = _ids(raw)
    out = np.empty(max(len(raw), 1), dtype=np.int64)
    m = lib().go_sort_unique(raw, len(raw), out)
    return out[:m].copy()


def feat_rows(seed: int, ids, dim: int, table: np.ndarray) -> np.ndarray:
    ids = _ids(ids)
    out = np.empty((len(ids), dim), dtype=table.dtype)
    table = np.ascontiguousarray(table)
    for i, v in enumerate(ids):
        lib().go_feat_row(seed, int(v), dim, table.dtype.itemsize, table.ctypes.data, out[i].ctypes.data)
    return out


def accum_threshold(iops_peak: float, t_initial: float, t_termination: float, ratio: float, n_ssd: int = 1) -> float:
    return float(lib().go_accum_threshold(iops_peak, t_initial, t_termination, ratio, n_ssd))


class Sim:
    """Batch-synchronous cache simulator.  `store` (a C-contiguous [n_rows, dim]
    array) switches on the data plane; without it only counts are produced."""

    def __init__(self, n_rows: int, lines: int, ways: int, window: int, row_bytes: int = 0, line_bytes: int = 0,
                 store: np.ndarray | None = None):
        self._store = None if store is None else np.ascontiguousarray(store)
        sp = None if store is None else self._store.ctypes.data
        self._h = lib().go_sim_create(n_rows, lines, ways, window, row_bytes, line_bytes, sp)
        if not self._h:
            raise OracleError(E_INVAL)
        self.n_rows, self.lines, self.ways, self.window = n_rows, lines, ways, window
        self.row_bytes = row_bytes

    def set_hot(self, ids) -> None:
        ids = _ids(ids)
        rc = lib().go_sim_set_hot(self._h, ids, len(ids))
        if rc:
            raise OracleError(rc)

    def set_policy(self, policy: int, seed: int = 0) -> None:
        """0 = LRU by minibatch (default), 1 = seeded random eviction"""
        rc = lib().go_sim_set_policy(self._h, policy, seed)
        if rc:
            raise OracleError(rc)

    def set_rows_per_line(self, rows: int) -> None:
        """cache lines hold `rows` consecutive node rows (default 1)"""
        rc = lib().go_sim_set_rows_per_line(self._h, rows)
        if rc:
            raise OracleError(rc)

    def set_accum(self, threshold: int, mode: int = 0) -> None:
        """storage access accumulator: merge minibatches until `threshold` node accesses (mode 0), or until
        the node accesses that bring `threshold` store accesses (mode 1)"""
        rc = lib().go_sim_set_accum(self._h, threshold, mode)
        if rc:
            raise OracleError(rc)

    def flush(self) -> int:
        """close the open group; returns the rows that were waiting"""
        return int(lib().go_sim_flush(self._h))

    @property
    def accum_last(self):
        """(rows pending after the latest gather, whether it closed its group, its node-access threshold)"""
        out = np.zeros(3, dtype=np.int64)
        lib().go_sim_accum_last(self._h, out)
        return int(out[0]), int(out[1]), int(out[2])

    def push(self, raw) -> None:
        raw = _ids(raw)
        rc = lib().go_sim_push(self._h, raw, len(raw))
        if rc:
            raise OracleError(rc)

    def gather(self, raw, want_rows: bool = True, want_cls: bool = False):
        """-> (unique int64[m], rows uint8[m, row_bytes] or None, stats int64[5][, cls int32[m]])"""
        raw = _ids(raw)
        n = len(raw)
        uniq = np.empty(max(n, 1), dtype=np.int64)
        stats = np.zeros(5, dtype=np.int64)
        rows = None
        if want_rows and self._store is not None:
            rows = np.empty((max(n, 1), self.row_bytes), dtype=np.uint8)
        cls = np.empty(max(n, 1), dtype=np.int32) if want_cls else None
        m = lib().go_sim_gather(self._h, raw, n, uniq, None if rows is None else rows.ctypes.data, stats,
                                None if cls is None else cls.ctypes.data)
        if m < 0:
            raise OracleError(int(m))
        res = (uniq[:m].copy(), None if rows is None else rows[:m], stats)
        return res + (cls[:m].copy(),) if want_cls else res

    @property
    def tags(self) -> np.ndarray:
        return np.ctypeslib.as_array(lib().go_sim_tags(self._h), shape=(self.lines,))

    @property
    def stamps(self) -> np.ndarray:
        return np.ctypeslib.as_array(lib().go_sim_stamps(self._h), shape=(self.lines,))

    @property
    def reuse(self) -> np.ndarray:
        return np.ctypeslib.as_array(lib().go_sim_reuse(self._h), shape=(self.n_rows,))

    @property
    def batch(self) -> int:
        return int(lib().go_sim_batch(self._h))

    @property
    def window_count(self) -> int:
        return int(lib().go_sim_window_count(self._h))

    def __del__(self):
        if getattr(self, "_h", None):
            lib().go_sim_free(self._h)
            self._h = None
