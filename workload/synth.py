"""Vectorised (numpy) generators for the synthetic GNN workload.

Everything here is a pure function of a 64-bit seed and integer counters, built
from one 64-bit mixing function, so that an independent implementation (the CPU
oracle has its own, written in C) reproduces every value bit for bit.

Definitions (all arithmetic modulo 2**64 unless stated):

  mix64(z):  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9; z ^= z >> 27;
             z *= 0x94D049BB133111EB; z ^= z >> 31
  H(seed, tag, x1, ..., xk):  k = mix64(seed + tag * 0x9E3779B97F4A7C15);
             then k = mix64(k ^ xi) for each xi in order

  degree(v)    x = ((H(seed, DEG, v) >> 32) + 1) / 2**32 in (0, 1];
               q = sqrt(sqrt(x)); y = q * q * ... (p4 factors);
               deg = clamp(floor(ell / y), 1, d_max)          (IEEE double)
               -> a bounded Pareto with tail exponent a - 1 = 4 / p4
  edge slot e  indices[e] = the node that owns edge slot (H(seed, EDGE, e) mod E)
               -> in-degree is proportional to out-degree
  seeds        seed_i of minibatch b = H(seed, SEED, b, i) mod N
  neighbours   node v at layer l of minibatch b with degree d and fanout f:
               d <= f: slots 0..d-1; otherwise f distinct slots by Floyd's
               subset sampling: for j = d-f .. d-1: t = H(seed, NBR, b, l, v, j)
               mod (j + 1); take t unless already taken, else take j
  features     feat(v, c) = T[(H(seed, FEAT, v, c >> 2) >> (16 * (c & 3))) & 0xFFFF]
               with T a 65536-entry table of N(0,1) quantiles in the row dtype

  layer-wise   (second workload, Section 4.7) layer l of minibatch b keeps a fixed
               number s_l of the distinct nodes that the adjacency slots of the
               previous layer point to: slot e gets key H(seed, LAYER, b, l, e), a
               node's key is the smallest key among the slots that point to it, and
               the s_l nodes of smallest key are kept (ties -> lower ID).  The
               minimum of m uniform keys wins with probability proportional to m,
               so this is weighted sampling without replacement, weight = number of
               connections into the previous layer

The sampling workload follows the two-layer neighbourhood sampling example of
the GraphSAGE description in Section 2.2.2 of the paper ("up to" fanout
neighbours per node, uniformly at random).
"""
from __future__ import annotations

import ctypes
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

U64 = np.uint64
GOLDEN = U64(0x9E3779B97F4A7C15)
M1 = U64(0xBF58476D1CE4E5B9)
M2 = U64(0x94D049BB133111EB)
TAGS = {"DEG": 1, "EDGE": 2, "FEAT": 3, "SEED": 4, "NBR": 5, "PERM": 6, "RANK": 7, "LAYER": 9}


def mix64(z):
    """The 64-bit finaliser every generator here is built from (vectorised)."""
    z = np.asarray(z, dtype=U64).copy()
    z ^= z >> U64(30)
    z *= M1
    z ^= z >> U64(27)
    z *= M2
    z ^= z >> U64(31)
    return z


def hash_chain(seed: int, tag: int, *xs):
    """H(seed, tag, x1..xk); each xi a scalar or an array (broadcast together)."""
    with np.errstate(over="ignore"):
        k = mix64(np.array((int(seed) + int(tag) * int(GOLDEN)) & 0xFFFFFFFFFFFFFFFF, dtype=U64))
        for x in xs:
            k = mix64(k ^ np.asarray(x).astype(U64))
    return k


@dataclass
class Graph:
    n: int
    indptr: np.ndarray   # int64[n + 1]
    indices: np.ndarray  # int64[E] (int32 when the config says so)
    seed: int

    @property
    def n_edges(self) -> int:
        return int(self.indptr[-1])

    def degrees(self) -> np.ndarray:
        return np.diff(self.indptr)


def degrees_for(seed: int, n: int, ell: float, p4: int, d_max: int, lo: int = 0, hi: int | None = None):
    hi = n if hi is None else hi
    v = np.arange(lo, hi, dtype=U64)
    h = hash_chain(seed, TAGS["DEG"], v)
    x = ((h >> U64(32)).astype(np.float64) + 1.0) / 4294967296.0
    q = np.sqrt(np.sqrt(x))
    y = q.copy()
    for _ in range(p4 - 1):
        y = y * q
    d = np.floor(ell / y)
    d = np.clip(d, 1.0, float(d_max))
    return d.astype(np.int64)


def _chunks(total: int, step: int):
    for lo in range(0, total, step):
        yield lo, min(total, lo + step)


def _threads() -> int:
    return max(1, min(16, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))))


def make_graph(seed: int, n: int, ell: float, p4: int, d_max: int | None = None,
               index_dtype=np.int64, chunk: int = 1 << 24, native: bool = False) -> Graph:
    """Power-law out-degrees, destinations proportional to out-degree, CSR.
    native=True computes the destinations with the multi-threaded C helper
    (same definition, for the multi-million-node configurations)."""
    if d_max is None:
        d_max = min(n - 1, 65535)
    indptr = np.zeros(n + 1, dtype=np.int64)
    with ThreadPoolExecutor(_threads()) as ex:
        parts = list(ex.map(lambda r: degrees_for(seed, n, ell, p4, d_max, r[0], r[1]), _chunks(n, 1 << 22)))
    np.cumsum(np.concatenate(parts), out=indptr[1:])
    del parts
    e_total = int(indptr[-1])
    indices = np.empty(e_total, dtype=index_dtype)
    if native:
        lib = _native_fill()
        lib.wl_make_edges(ctypes.c_uint64(seed), ctypes.c_int64(n), indptr.ctypes.data_as(ctypes.c_void_p),
                          ctypes.c_int64(0), ctypes.c_int64(e_total), indices.ctypes.data_as(ctypes.c_void_p),
                          ctypes.c_uint32(indices.dtype.itemsize), ctypes.c_int(_threads()))
        return Graph(n=n, indptr=indptr, indices=indices, seed=seed)

    def work(rng):
        lo, hi = rng
        h = hash_chain(seed, TAGS["EDGE"], np.arange(lo, hi, dtype=U64))
        slot = (h % U64(e_total)).astype(np.int64)
        indices[lo:hi] = np.searchsorted(indptr, slot, side="right") - 1

    with ThreadPoolExecutor(_threads()) as ex:
        list(ex.map(work, _chunks(e_total, chunk)))
    return Graph(n=n, indptr=indptr, indices=indices, seed=seed)


def hot_nodes(g: Graph, k: int) -> np.ndarray:
    """IDs of the k nodes with the largest in-degree (ties: lower ID first)."""
    if k <= 0:
        return np.empty(0, dtype=np.int64)
    indeg = np.bincount(g.indices, minlength=g.n).astype(np.int64)
    if k < g.n // 4:
        # only nodes at or above the k-th largest in-degree can be in the answer
        kth = np.partition(indeg, g.n - k)[g.n - k]
        cand = np.flatnonzero(indeg >= kth).astype(np.int64)
    else:
        cand = np.arange(g.n, dtype=np.int64)
    order = np.lexsort((cand, -indeg[cand]))
    return cand[order[:k]]


def top_k_by_score(score: np.ndarray, k: int) -> np.ndarray:
    """IDs of the k largest scores (ties: lower ID first)."""
    n = len(score)
    if k <= 0:
        return np.empty(0, dtype=np.int64)
    if k < n // 4:
        kth = np.partition(score, n - k)[n - k]
        cand = np.flatnonzero(score >= kth).astype(np.int64)
    else:
        cand = np.arange(n, dtype=np.int64)
    sc = score[cand]
    order = np.lexsort((cand, sc.max() - sc))
    return cand[order[:k]]


def zipf_rank_table(n: int, s: float) -> np.ndarray:
    """Cumulative thresholds (uint64, scaled to 2**63) of Zipf(s) over ranks 1..n."""
    w = np.arange(1, n + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(w)
    c /= c[-1]
    t = np.floor(c * float(1 << 63)).astype(U64)
    t[-1] = U64(1 << 63)
    return t


def minibatch_seeds(seed: int, n: int, batch: int, n_seeds: int, rank_table: np.ndarray | None = None):
    """Seed nodes of minibatch `batch`: uniform with replacement, or Zipf-ranked.

    With a rank table the draw picks rank r by inverse CDF over the integer
    thresholds and maps it to node (r * PERM_MULT + PERM_ADD) mod n with the
    seeded odd multiplier / offset below (a fixed bijection when gcd(mult, n) = 1).
    """
    i = np.arange(n_seeds, dtype=U64)
    h = hash_chain(seed, TAGS["SEED"], batch, i)
    if rank_table is None:
        return (h % U64(n)).astype(np.int64)
    u = h >> U64(1)
    r = np.searchsorted(rank_table, u, side="right").astype(np.int64)
    r = np.minimum(r, n - 1)
    mult, add = perm_params(seed, n)
    return np.array([(int(x) * mult + add) % n for x in r], dtype=np.int64)


def perm_params(seed: int, n: int):
    """Multiplier coprime to n and an offset, both from the seed."""
    from math import gcd
    k = int(hash_chain(seed, TAGS["PERM"], 0))
    mult = (k % n) | 1
    while gcd(mult, n) != 1:
        mult += 2
    add = int(hash_chain(seed, TAGS["PERM"], 1)) % n
    return mult, add


def sample_minibatch(g: Graph, seed: int, batch: int, fanouts, n_seeds: int,
                     rank_table: np.ndarray | None = None) -> np.ndarray:
    """Raw node-ID list of one minibatch: seeds, then each layer's sampled
    neighbours in frontier order (ascending node, chosen slots in draw order),
    duplicates kept.  Each hop expands the distinct nodes the previous hop
    reached (the seeds for the first hop)."""
    seeds = minibatch_seeds(seed, g.n, batch, n_seeds, rank_table)
    parts = [seeds]
    frontier = np.unique(seeds)
    indptr, indices = g.indptr, g.indices
    for layer, f in enumerate(fanouts):
        start = indptr[frontier]
        deg = indptr[frontier + 1] - start
        take = np.minimum(deg, f)
        out_off = np.zeros(len(frontier) + 1, dtype=np.int64)
        np.cumsum(take, out=out_off[1:])
        slots = np.empty(int(out_off[-1]), dtype=np.int64)
        small = deg <= f
        # all slots of small-degree nodes
        if small.any():
            cnt = take[small]
            base = np.repeat(out_off[:-1][small], cnt)
            within = np.arange(int(cnt.sum()), dtype=np.int64) - np.repeat(np.cumsum(cnt) - cnt, cnt)
            slots[base + within] = within
        big = ~small
        if big.any():
            vb = frontier[big].astype(U64)
            db = deg[big]
            kv = hash_chain(seed, TAGS["NBR"], batch, layer, vb)
            chosen = np.empty((len(vb), f), dtype=np.int64)
            for k in range(f):
                j = db - f + k
                with np.errstate(over="ignore"):
                    t = (mix64(kv ^ j.astype(U64)) % (j + 1).astype(U64)).astype(np.int64)
                if k:
                    dup = (chosen[:, :k] == t[:, None]).any(axis=1)
                    t = np.where(dup, j, t)
                chosen[:, k] = t
            pos = out_off[:-1][big][:, None] + np.arange(f, dtype=np.int64)[None, :]
            slots[pos.ravel()] = chosen.ravel()
        src = np.repeat(start, take) + slots
        sampled = indices[src].astype(np.int64)
        parts.append(sampled)
        frontier = np.unique(sampled)
    return np.concatenate(parts)


def layerwise_minibatch(g: Graph, seed: int, batch: int, layer_sizes, n_seeds: int) -> np.ndarray:
    """Raw node-ID list of one minibatch under layer-wise sampling: the seeds, then
    for each layer a fixed number of nodes drawn from the neighbourhood of the
    previous layer with probability proportional to how many of its adjacency
    slots point to them (ascending ID order within a layer)."""
    seeds = minibatch_seeds(seed, g.n, batch, n_seeds)
    parts = [seeds]
    cur = np.unique(seeds)
    indptr, indices = g.indptr, g.indices
    for layer, size in enumerate(layer_sizes):
        start = indptr[cur]
        deg = indptr[cur + 1] - start
        total = int(deg.sum())
        if total == 0:
            break
        slot = np.repeat(start, deg) + (np.arange(total, dtype=np.int64) - np.repeat(np.cumsum(deg) - deg, deg))
        nbr = indices[slot].astype(np.int64)
        key = hash_chain(seed, TAGS["LAYER"], batch, layer, slot.astype(U64))
        # Only the slots of smallest key can decide: look at a prefix of the key order first.
        look = min(total, 4 * size + 1024)
        while True:
            if look < total:
                part = np.argpartition(key, look - 1)[:look]
                nbr_p, key_p = nbr[part], key[part]
                bound = key_p.max()                          # every slot outside the prefix has a key >= bound
            else:
                nbr_p, key_p, bound = nbr, key, None
            order = np.lexsort((key_p, nbr_p))               # by node, then key: first of each node = its smallest
            nbr_s, key_s = nbr_p[order], key_p[order]
            first = np.concatenate([[True], nbr_s[1:] != nbr_s[:-1]])
            cand, ckey = nbr_s[first], key_s[first]
            keep = np.lexsort((cand, ckey))[:size]           # smallest keys, ties -> lower ID
            # complete when no slot outside the prefix could beat or tie the last one kept
            if bound is None or (len(keep) == size and ckey[keep[-1]] < bound):
                break
            look = min(total, look * 4)
        chosen = np.sort(cand[keep])
        parts.append(chosen)
        cur = chosen
    return np.concatenate(parts)


def normal_table(dtype) -> np.ndarray:
    """T[i] = the N(0,1) quantile at (i + 0.5) / 65536, rounded to `dtype`."""
    from scipy.special import ndtri
    p = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
    return ndtri(p).astype(dtype)


def feature_rows(seed: int, ids, dim: int, table: np.ndarray) -> np.ndarray:
    """Rows feat(v, 0..dim-1) for the given node IDs (dim a multiple of 4)."""
    ids = np.asarray(ids, dtype=U64)
    assert dim % 4 == 0
    kv = hash_chain(seed, TAGS["FEAT"], ids)
    g = np.arange(dim // 4, dtype=U64)
    with np.errstate(over="ignore"):
        w = mix64(kv[:, None] ^ g[None, :])
    idx = np.empty((len(ids), dim // 4, 4), dtype=np.uint16)
    for q in range(4):
        idx[:, :, q] = ((w >> U64(16 * q)) & U64(0xFFFF)).astype(np.uint16)
    return table[idx.reshape(len(ids), dim)]


_fill_lib = None


def _native_fill():
    """Optional multi-threaded C filler (same closed form), built on demand."""
    global _fill_lib
    if _fill_lib is None:
        from . import native
        _fill_lib = native.load()
    return _fill_lib


def fill_store(seed: int, n_rows: int, dim: int, table: np.ndarray, out: np.ndarray | int,
               row_lo: int = 0, native: bool = True, threads: int | None = None) -> None:
    """Write rows row_lo .. row_lo + n_rows - 1 of the feature table into `out`
    (an array of shape [n_rows, dim] or a raw address of that many bytes)."""
    itemsize = table.dtype.itemsize
    if native:
        lib = _native_fill()
        addr = out if isinstance(out, int) else out.ctypes.data
        lib.wl_fill_store(ctypes.c_uint64(seed), ctypes.c_uint64(row_lo), ctypes.c_uint64(n_rows),
                          ctypes.c_uint32(dim), ctypes.c_uint32(itemsize),
                          table.ctypes.data_as(ctypes.c_void_p), ctypes.c_void_p(addr),
                          ctypes.c_int(threads or _threads()))
        return
    assert not isinstance(out, int)
    step = max(1, (1 << 22) // dim)
    for lo, hi in _chunks(n_rows, step):
        out[lo:hi] = feature_rows(seed, np.arange(row_lo + lo, row_lo + hi), dim, table)
