"""ctypes binding of libgids.so: the C ABI of include/gids.h under the same
names, argument marshalling only.  Every step of the gather runs in the HIP
kernels of the library; there is no fallback, a missing library is an error."""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgids.so")

GIDS_OK = 0
GIDS_E_INVAL, GIDS_E_NOMEM, GIDS_E_RANGE, GIDS_E_ORDER, GIDS_E_FULL, GIDS_E_HIP, GIDS_E_SPACE = -1, -2, -3, -4, -5, -6, -7

EXPORTS = [
    "gids_store_create", "gids_store_host_ptr", "gids_store_destroy", "gids_store_calibrate", "gids_cache_create", "gids_cache_destroy",
    "gids_cache_reserve", "gids_cache_set_policy", "gids_cache_set_accum_mode", "gids_cache_set_group_dedup", "gids_cpu_buffer_pin", "gids_window_push", "gids_gather", "gids_gather_static", "gids_gather_many", "gids_flush", "gids_stats_read",
    "gids_cache_gathers", "gids_cache_many_calls", "gids_cache_snapshot", "gids_cache_set_rows_per_line", "gids_profile_enable", "gids_profile_read", "gids_window_push_dev",
    "gids_graph_create", "gids_graph_destroy", "gids_sample_capacity", "gids_sample", "gids_graph_visit_scores", "gids_graph_reverse_pagerank", "gids_accum_threshold", "gids_last_error",
]


class gids_stats(C.Structure):
    _fields_ = [("seq", C.c_uint64), ("n_unique", C.c_uint64), ("n_hit", C.c_uint64), ("n_cpu_hit", C.c_uint64),
                ("n_miss", C.c_uint64), ("n_bypass", C.c_uint64), ("n_pending", C.c_uint64),
                ("flushed", C.c_int32), ("status", C.c_int32), ("n_line_fills", C.c_uint64), ("n_cpu_again", C.c_uint64)]

    def as_tuple(self):
        """(n_unique, hits, CPU-buffer hits, misses, bypasses)"""
        return (self.n_unique, self.n_hit, self.n_cpu_hit, self.n_miss, self.n_bypass)


class GidsError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"gids error {code}: {text}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2306_16384_amd.build` "
                               "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        vp, u64, u32 = C.c_void_p, C.c_uint64, C.c_uint32
        L.gids_store_create.argtypes = [u64, u32, u32, vp, C.POINTER(vp)]
        L.gids_store_host_ptr.restype = vp
        L.gids_store_host_ptr.argtypes = [vp]
        L.gids_store_destroy.argtypes = [vp]
        L.gids_store_calibrate.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.gids_cache_create.argtypes = [vp, u64, u32, u32, u32, u64, C.POINTER(vp)]
        L.gids_cache_destroy.argtypes = [vp]
        L.gids_cache_reserve.argtypes = [vp, u64]
        L.gids_cache_set_policy.argtypes = [vp, C.c_int, u64]
        L.gids_cache_set_rows_per_line.argtypes = [vp, u32]
        L.gids_cache_set_accum_mode.argtypes = [vp, C.c_int]
        L.gids_cache_set_group_dedup.argtypes = [vp, C.c_int]
        L.gids_cpu_buffer_pin.argtypes = [vp, vp, u64]
        L.gids_window_push.argtypes = [vp, vp, u64, vp]
        L.gids_gather.argtypes = [vp, vp, u64, vp, u64, vp, vp, vp]
        L.gids_gather_static.argtypes = [vp, vp, u64, vp, u64, vp, vp]
        L.gids_gather_many.argtypes = [vp, u32, C.POINTER(vp), C.POINTER(u64), C.POINTER(vp), C.POINTER(u64), C.POINTER(vp), vp, vp]
        L.gids_flush.argtypes = [vp, vp]
        L.gids_stats_read.argtypes = [vp, u64, C.POINTER(gids_stats)]
        L.gids_cache_gathers.restype = u64
        L.gids_cache_gathers.argtypes = [vp]
        L.gids_cache_many_calls.restype = None
        L.gids_cache_many_calls.argtypes = [vp, C.POINTER(u64), C.POINTER(u64)]
        L.gids_cache_snapshot.argtypes = [vp, vp, vp]
        L.gids_window_push_dev.argtypes = [vp, vp, u64, vp, vp]
        L.gids_graph_create.argtypes = [u64, vp, vp, u32, C.c_int, C.POINTER(vp)]
        L.gids_graph_destroy.argtypes = [vp]
        L.gids_sample_capacity.restype = u64
        L.gids_sample_capacity.argtypes = [C.POINTER(u32), u32, u64]
        L.gids_sample.argtypes = [vp, u64, u64, C.POINTER(u32), u32, u64, vp, u64, u64, vp, u64, vp, vp]
        L.gids_graph_visit_scores.argtypes = [vp, C.POINTER(u32), u32, u64, vp, vp]
        L.gids_graph_reverse_pagerank.argtypes = [vp, u32, u32, vp, vp]
        L.gids_profile_enable.argtypes = [vp, C.c_int]
        L.gids_profile_read.argtypes = [vp, u64, C.POINTER(C.c_float)]
        L.gids_accum_threshold.restype = C.c_double
        L.gids_accum_threshold.argtypes = [C.c_double, C.c_double, C.c_double, C.c_double, C.c_int]
        L.gids_last_error.restype = C.c_char_p
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != GIDS_OK:
        raise GidsError(rc, lib().gids_last_error().decode())


def gids_store_create(n_rows: int, row_bytes: int, id_bytes: int, host_ptr: int | None = None) -> int:
    h = C.c_void_p()
    _check(lib().gids_store_create(n_rows, row_bytes, id_bytes, host_ptr, C.byref(h)))
    return h.value


def gids_store_host_ptr(store: int) -> int:
    return lib().gids_store_host_ptr(store)


def gids_store_calibrate(store: int):
    """-> (rows per second over the link, fixed overhead in seconds)"""
    rate, over = C.c_double(), C.c_double()
    _check(lib().gids_store_calibrate(store, C.byref(rate), C.byref(over)))
    return rate.value, over.value


def gids_store_destroy(store: int) -> None:
    _check(lib().gids_store_destroy(store))


def gids_cache_create(store: int, lines: int, ways: int, line_bytes: int, window_depth: int = 0,
                      accum_threshold: int = 0) -> int:
    h = C.c_void_p()
    _check(lib().gids_cache_create(store, lines, ways, line_bytes, window_depth, accum_threshold, C.byref(h)))
    return h.value


def gids_cache_destroy(cache: int) -> None:
    _check(lib().gids_cache_destroy(cache))


def gids_cache_reserve(cache: int, max_ids: int) -> None:
    _check(lib().gids_cache_reserve(cache, max_ids))


GIDS_POLICY_LRU, GIDS_POLICY_RANDOM = 0, 1


def gids_cache_set_policy(cache: int, policy: int, seed: int = 0) -> None:
    _check(lib().gids_cache_set_policy(cache, policy, seed))


GIDS_ACCUM_FIXED, GIDS_ACCUM_ADAPTIVE = 0, 1
GIDS_ACCUM_MAX_MERGE, GIDS_ACCUM_LAG, GIDS_ACCUM_MAX_RAISE = 32, 16, 8


def gids_cache_set_accum_mode(cache: int, mode: int) -> None:
    _check(lib().gids_cache_set_accum_mode(cache, mode))


def gids_cache_set_group_dedup(cache: int, on: bool) -> None:
    _check(lib().gids_cache_set_group_dedup(cache, 1 if on else 0))


def gids_cache_set_rows_per_line(cache: int, rows: int) -> None:
    _check(lib().gids_cache_set_rows_per_line(cache, rows))


def gids_cpu_buffer_pin(cache: int, ids_host_ptr: int, n: int) -> None:
    _check(lib().gids_cpu_buffer_pin(cache, ids_host_ptr, n))


def gids_window_push(cache: int, ids_dev_ptr: int, n: int, stream: int = 0) -> None:
    _check(lib().gids_window_push(cache, ids_dev_ptr, n, stream))


def gids_gather(cache: int, ids_dev_ptr: int | None, n: int, out_dev_ptr: int, out_capacity_rows: int,
                unique_dev_ptr: int | None = None, inverse_dev_ptr: int | None = None, stream: int = 0) -> None:
    _check(lib().gids_gather(cache, ids_dev_ptr, n, out_dev_ptr, out_capacity_rows, unique_dev_ptr, inverse_dev_ptr,
                             stream))


GIDS_STATIC_MAX_IDS = 1 << 20


def gids_gather_static(cache: int, ids_dev_ptr: int | None, n: int, out_dev_ptr: int, out_capacity_rows: int,
                       unique_dev_ptr: int | None = None, stream: int = 0) -> None:
    _check(lib().gids_gather_static(cache, ids_dev_ptr, n, out_dev_ptr, out_capacity_rows, unique_dev_ptr, stream))


def gids_gather_many(cache: int, push_ids_dev_ptrs, push_n, out_dev_ptrs, out_capacity_rows, unique_dev_ptrs=None,
                     push_stream: int = 0, stream: int = 0) -> None:
    """k steps (push one list or None, gather the window's head) in one call; sequences of k entries"""
    k = len(out_dev_ptrs)
    vp_k, u64_k = C.c_void_p * k, C.c_uint64 * k
    pushes = None if push_ids_dev_ptrs is None else vp_k(*push_ids_dev_ptrs)
    lens = None if push_ids_dev_ptrs is None else u64_k(*[int(x) for x in push_n])
    uniq = None if unique_dev_ptrs is None else vp_k(*unique_dev_ptrs)
    _check(lib().gids_gather_many(cache, k, pushes, lens, vp_k(*out_dev_ptrs), u64_k(*[int(x) for x in out_capacity_rows]),
                                  uniq, push_stream, stream))


def gids_flush(cache: int, stream: int = 0) -> None:
    _check(lib().gids_flush(cache, stream))


def gids_stats_read(cache: int, seq: int) -> gids_stats:
    st = gids_stats()
    _check(lib().gids_stats_read(cache, seq, C.byref(st)))
    return st


def gids_cache_gathers(cache: int) -> int:
    return int(lib().gids_cache_gathers(cache))


def gids_cache_many_calls(cache: int) -> tuple[int, int]:
    """(calls through the merged kernels, calls through the per-step kernels)"""
    a, b = C.c_uint64(0), C.c_uint64(0)
    lib().gids_cache_many_calls(cache, C.byref(a), C.byref(b))
    return int(a.value), int(b.value)


def gids_cache_snapshot(cache: int, tags_host_ptr: int | None, stamps_host_ptr: int | None) -> None:
    _check(lib().gids_cache_snapshot(cache, tags_host_ptr, stamps_host_ptr))


def gids_window_push_dev(cache: int, ids_dev_ptr: int, n_max: int, n_dev_ptr: int, stream: int = 0) -> None:
    _check(lib().gids_window_push_dev(cache, ids_dev_ptr, n_max, n_dev_ptr, stream))


def gids_graph_create(n_nodes: int, indptr_host_ptr: int, indices_host_ptr: int, id_bytes: int,
                      zero_copy: bool = False) -> int:
    h = C.c_void_p()
    _check(lib().gids_graph_create(n_nodes, indptr_host_ptr, indices_host_ptr, id_bytes, 1 if zero_copy else 0,
                                   C.byref(h)))
    return h.value


def gids_graph_destroy(graph: int) -> None:
    _check(lib().gids_graph_destroy(graph))


def _fanouts(fanouts):
    arr = (C.c_uint32 * len(fanouts))(*[int(f) for f in fanouts])
    return arr, len(fanouts)


def gids_sample_capacity(fanouts, n_seeds: int) -> int:
    arr, n = _fanouts(fanouts)
    return int(lib().gids_sample_capacity(arr, n, n_seeds))


def gids_sample(graph: int, seed: int, batch: int, fanouts, n_seeds: int, raw_dev_ptr: int, raw_capacity: int,
                n_raw_dev_ptr: int, stream: int = 0, rank_table_dev_ptr: int | None = None, perm_mult: int = 0,
                perm_add: int = 0) -> None:
    arr, n = _fanouts(fanouts)
    _check(lib().gids_sample(graph, seed, batch, arr, n, n_seeds, rank_table_dev_ptr, perm_mult, perm_add, raw_dev_ptr,
                             raw_capacity, n_raw_dev_ptr, stream))


def gids_graph_visit_scores(graph: int, fanouts, n_seeds: int, scores_dev_ptr: int, stream: int = 0) -> None:
    arr, n = _fanouts(fanouts)
    _check(lib().gids_graph_visit_scores(graph, arr, n, n_seeds, scores_dev_ptr, stream))


def gids_graph_reverse_pagerank(graph: int, damping_q16: int, n_iters: int, scores_dev_ptr: int, stream: int = 0) -> None:
    _check(lib().gids_graph_reverse_pagerank(graph, damping_q16, n_iters, scores_dev_ptr, stream))


def gids_profile_enable(cache: int, on: bool) -> None:
    _check(lib().gids_profile_enable(cache, 1 if on else 0))


def gids_profile_read(cache: int, seq: int):
    """-> (dedup ms, probe + victim ms, row movement ms) of gather `seq`"""
    ms = (C.c_float * 3)()
    _check(lib().gids_profile_read(cache, seq, ms))
    return tuple(float(x) for x in ms)


def gids_accum_threshold(iops_peak: float, t_initial: float, t_termination: float, ratio: float, n_ssd: int = 1) -> float:
    return float(lib().gids_accum_threshold(iops_peak, t_initial, t_termination, ratio, n_ssd))


def gids_last_error() -> str:
    return lib().gids_last_error().decode()
