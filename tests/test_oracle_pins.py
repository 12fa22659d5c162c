"""Pins of the CPU oracle against what the paper and the mathematics fix.

Each test checks the oracle against something other than itself: the plain
definition of a gather, a set-based dedup, an independently written textbook
LRU, brute force over the future ID lists, closed forms, a hand-traced table,
and the numbers of the paper's worked examples."""
from collections import OrderedDict

import numpy as np
import pytest

import os

import workload as wl
from workload import CONFIGS

GOLDEN = {}
with open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")) as fh:
    for line in fh:
        if line.strip() and not line.startswith("#"):
            k, v = line.split("#")[0].split("=")
            GOLDEN[k.strip()] = float(v)


# ------------------------------------------------------------------ helpers

def tiny_setup(oracle, n=400, dim=8, lines=32, ways=4, window=2, n_hot=10, seed=3, store=True):
    rng = np.random.default_rng(seed)
    feats = rng.standard_normal((n, dim)).astype(np.float32)
    sim = oracle.Sim(n, lines, ways, window, dim * 4, dim * 4, feats if store else None)
    hot = rng.choice(n, size=n_hot, replace=False).astype(np.int64)
    if n_hot:
        sim.set_hot(hot)
    return rng, feats, sim, hot


def run_stream(sim, batches, window):
    """Push `window` + 1 lists ahead, gather in order; returns per-batch results."""
    res = []
    pushed = 0
    for t in range(len(batches)):
        while window and pushed < len(batches) and pushed <= t + window:
            sim.push(batches[pushed])
            pushed += 1
        res.append(sim.gather(batches[t], want_cls=True))
    return res


def zipf_batches(rng, n, n_batches, size, a=1.3):
    out = []
    for _ in range(n_batches):
        out.append(np.minimum(rng.zipf(a, size=size) - 1, n - 1).astype(np.int64))
    return out


# ------------------------------------------------- the plain definitions

def test_sort_unique_vs_set(oracle_mod):
    rng = np.random.default_rng(0)
    for n in (0, 1, 2, 17, 1000):
        raw = rng.integers(0, 50, size=n)
        want = np.array(sorted(set(raw.tolist())), dtype=np.int64)
        np.testing.assert_array_equal(oracle_mod.sort_unique(raw), want)


@pytest.mark.parametrize("window", [0, 3])
def test_rows_equal_store_rows_brute_force(oracle_mod, window):
    """Section 2.2.3: the gather returns, for every distinct ID, that node's feature row."""
    rng, feats, sim, hot = tiny_setup(oracle_mod, window=window)
    batches = zipf_batches(rng, 400, 25, 120)
    for (uniq, rows, stats, cls), raw in zip(run_stream(sim, batches, window), batches):
        want_ids = sorted(set(raw.tolist()))
        assert uniq.tolist() == want_ids
        for j, v in enumerate(want_ids):                   # row by row, the definition itself
            assert rows[j].tobytes() == feats[v].tobytes()
        assert stats[0] == len(want_ids)
        assert stats[1] + stats[2] + stats[3] == stats[0]  # hits + CPU-buffer hits + misses = unique IDs
        assert stats[4] <= stats[3]
        assert np.sum(cls == oracle_mod.CLS_HIT) == stats[1]
        assert np.sum(cls == oracle_mod.CLS_CPU) == stats[2]
        assert np.sum((cls == oracle_mod.CLS_MISS) | (cls == oracle_mod.CLS_BYPASS)) == stats[3]
        assert np.sum(cls == oracle_mod.CLS_BYPASS) == stats[4]


def test_cpu_buffer_hits_closed_form(oracle_mod):
    """Section 3.3: an ID pinned in the CPU buffer is always served from it, whatever the cache holds."""
    rng, feats, sim, hot = tiny_setup(oracle_mod, n_hot=40, window=2)
    batches = zipf_batches(rng, 400, 20, 150)
    hotset = set(hot.tolist())
    for (uniq, rows, stats, cls), raw in zip(run_stream(sim, batches, 2), batches):
        assert stats[2] == len(set(raw.tolist()) & hotset)
        assert all((c == oracle_mod.CLS_CPU) == (v in hotset) for v, c in zip(uniq.tolist(), cls.tolist()))
    assert not (set(sim.tags.tolist()) & hotset)           # hot rows never enter the GPU cache


def test_permutation_and_duplication_invariance(oracle_mod):
    rng = np.random.default_rng(5)
    batches = zipf_batches(rng, 300, 12, 90)
    runs = []
    for variant in range(3):
        sim = oracle_mod.Sim(300, 24, 4, 2)
        sim.set_hot(np.arange(0, 300, 37))
        bs = []
        for b in batches:
            if variant == 1:
                b = rng.permutation(b)
            elif variant == 2:
                b = np.concatenate([b, b[::3], b[:5]])
            bs.append(b)
        runs.append([(u.tolist(), s.tolist(), c.tolist()) for u, _, s, c in run_stream(sim, bs, 2)])
    assert runs[0] == runs[1] == runs[2]


# ------------------------------------------------------ cache >= store

@pytest.mark.parametrize("window", [0, 4])
def test_cache_as_large_as_store_misses_only_first_touch(oracle_mod, window):
    n, ways = 240, 4
    n_sets = 60                                            # ceil(n / n_sets) = 4 = ways: modulo sets never overflow
    sim = oracle_mod.Sim(n, n_sets * ways, ways, window)
    rng = np.random.default_rng(1)
    batches = [rng.integers(0, n, size=70) for _ in range(40)]
    seen = set()
    total_miss = 0
    for (uniq, _, stats, cls), raw in zip(run_stream(sim, batches, window), batches):
        first = set(uniq.tolist()) - seen
        assert stats[3] == len(first) and stats[4] == 0    # a miss only on a node's first touch, never a bypass
        assert stats[1] == len(uniq) - len(first)
        seen |= first
        total_miss += stats[3]
    assert total_miss == len(seen)
    assert sorted(t for t in sim.tags.tolist() if t >= 0) == sorted(seen)


# ---------------------------------------------- window depth 0 == LRU

def test_depth0_single_id_batches_is_textbook_lru(oracle_mod):
    """With one ID per minibatch, least-recently-used-by-batch is exactly LRU."""
    n, n_sets, ways = 200, 4, 3
    sim = oracle_mod.Sim(n, n_sets * ways, ways, 0)
    lru = [OrderedDict() for _ in range(n_sets)]
    rng = np.random.default_rng(2)
    for v in np.minimum(rng.zipf(1.2, size=3000) - 1, n - 1):
        _, _, stats, _ = sim.gather(np.array([v]), want_cls=True)
        d = lru[v % n_sets]
        if v in d:
            d.move_to_end(v)
            want_hit = 1
        else:
            if len(d) == ways:
                d.popitem(last=False)
            d[v] = True
            want_hit = 0
        assert stats[1] == want_hit and stats[3] == 1 - want_hit
    for s in range(n_sets):
        assert set(sim.tags[s * ways:(s + 1) * ways].tolist()) - {-1} == set(int(k) for k in lru[s])


class BatchLRU:
    """Independent model of LRU-by-batch for multi-ID minibatches: per set a
    list of resident IDs ordered from least to most recently used, where all
    IDs touched by one minibatch count as used at the same time and ties are
    ordered by way index; IDs touched in the current minibatch are not victims."""

    def __init__(self, n_sets, ways):
        self.n_sets, self.ways = n_sets, ways
        self.way_of = [dict() for _ in range(n_sets)]       # id -> way
        self.last = [dict() for _ in range(n_sets)]         # id -> last batch
        self.t = 0

    def gather(self, ids):
        hits = misses = bypass = 0
        ids = sorted(set(ids))
        missing = {}
        for v in ids:
            s = v % self.n_sets
            if v in self.way_of[s]:
                hits += 1
                self.last[s][v] = self.t
            else:
                missing.setdefault(s, []).append(v)
        for s, vs in missing.items():
            free = [w for w in range(self.ways) if w not in self.way_of[s].values()]
            old = sorted((self.last[s][v], self.way_of[s][v], v) for v in self.way_of[s] if self.last[s][v] != self.t)
            victims = [(w, None) for w in free] + [(w, v) for _, w, v in old]
            for k, v in enumerate(vs):
                misses += 1
                if k < len(victims):
                    w, gone = victims[k]
                    if gone is not None:
                        del self.way_of[s][gone], self.last[s][gone]
                    self.way_of[s][v] = w
                    self.last[s][v] = self.t
                else:
                    bypass += 1
        self.t += 1
        return len(ids), hits, misses, bypass


def test_depth0_multi_id_batches_vs_independent_model(oracle_mod):
    n, n_sets, ways = 500, 8, 4
    sim = oracle_mod.Sim(n, n_sets * ways, ways, 0)
    model = BatchLRU(n_sets, ways)
    rng = np.random.default_rng(4)
    for raw in zipf_batches(rng, n, 60, 40, a=1.15):
        _, _, stats, _ = sim.gather(raw, want_cls=True)
        u, h, m, b = model.gather(raw.tolist())
        assert (stats[0], stats[1], stats[3], stats[4]) == (u, h, m, b)
    for s in range(n_sets):
        for v, w in model.way_of[s].items():
            assert sim.tags[s * ways + w] == v


# ------------------------------------------------------------- window

def test_window_never_evicts_a_line_with_a_buffered_future_use(oracle_mod):
    """Section 3.4: a cached node that one of the buffered future minibatches
    reuses stays in the 'USE' state and is not evicted."""
    n, lines, ways, window = 300, 32, 4, 3
    rng = np.random.default_rng(9)
    batches = zipf_batches(rng, n, 50, 60, a=1.2)
    usets = [set(b.tolist()) for b in batches]
    sim = oracle_mod.Sim(n, lines, ways, window)
    pushed, evicted_any = 0, 0
    for t in range(len(batches)):
        while pushed < len(batches) and pushed <= t + window:
            sim.push(batches[pushed])
            pushed += 1
        before = set(sim.tags.tolist()) - {-1}
        sim.gather(batches[t], want_rows=False)
        after = set(sim.tags.tolist()) - {-1}
        future = set().union(*usets[t + 1:t + 1 + window]) if t + 1 < len(batches) else set()
        gone = before - after
        evicted_any += len(gone)
        assert not (gone & future), (t, gone & future)
        assert not (gone & usets[t])                        # nor a line used by this very minibatch
        # the per-node counter is the number of buffered future minibatches that contain the node
        reuse = sim.reuse
        for v in range(n):
            assert reuse[v] == sum(v in u for u in usets[t + 1:pushed])
    assert evicted_any > 0


def test_window_raises_hit_count_on_a_cyclic_stream(oracle_mod):
    """A stream that cycles through more lines than one set holds thrashes LRU
    completely; with look-ahead the lines reused soonest are kept."""
    n, ways = 64, 4
    cycle = [np.array([v]) for v in range(0, 6)] * 12       # 6 IDs, one set of 4 ways
    hits = {}
    for window in (0, 4):
        sim = oracle_mod.Sim(n, ways, ways, window)
        hits[window] = sum(int(r[2][1]) for r in run_stream(sim, cycle, window))
    assert hits[0] == 0
    assert hits[4] > 20


# -------------------------------------------------- hand-traced table

def test_hand_traced_fully_associative_case(oracle_mod):
    """One set of four ways, look-ahead of two minibatches, node 7 in the CPU
    buffer; expected tags / stamps / counts worked out by hand from the rules:
    classify against the state at the start, USE lines (future count > 0) and
    lines touched in this minibatch are not victims, victims in (stamp, way)
    order go to the misses in ascending ID order, the rest bypass."""
    sim = oracle_mod.Sim(50, 4, 4, 2)
    sim.set_hot(np.array([7]))
    B = [[3, 1, 2, 7, 1], [5, 2, 4], [9, 8, 6, 1], [10, 3, 2, 2], [11, 1], [13, 12]]
    trace = []

    def g(i):
        _, _, st, _ = sim.gather(np.array(B[i]), want_cls=True)
        trace.append((st.tolist(), sim.tags.tolist(), sim.stamps.tolist()))

    for i in (0, 1, 2):
        sim.push(np.array(B[i]))
    g(0); sim.push(np.array(B[3]))
    g(1); sim.push(np.array(B[4]))
    g(2); sim.push(np.array(B[5]))
    g(3); g(4); g(5)
    want = [
        ([4, 0, 1, 3, 0], [1, 2, 3, -1], [0, 0, 0, -1]),
        ([3, 1, 0, 2, 1], [1, 2, 3, 4], [0, 1, 0, 1]),      # 1 and 3 are USE, 5 bypasses
        ([4, 1, 0, 3, 2], [1, 2, 3, 6], [2, 1, 0, 2]),      # only way 3 (node 4) is safe to evict
        ([3, 2, 0, 1, 0], [1, 2, 3, 10], [2, 3, 3, 3]),
        ([2, 1, 0, 1, 0], [1, 11, 3, 10], [4, 4, 3, 3]),    # three ways tie on stamp 3: lowest way goes
        ([2, 0, 0, 2, 0], [1, 11, 12, 13], [4, 4, 5, 5]),   # oldest stamps first
    ]
    assert trace == want


# --------------------------------------------------------------- errors

def test_protocol_errors(oracle_mod):
    sim = oracle_mod.Sim(20, 4, 2, 1)
    with pytest.raises(oracle_mod.OracleError) as e:
        sim.gather(np.array([1]))
    assert e.value.code == oracle_mod.E_ORDER                # nothing buffered
    sim.push(np.array([1, 2]))
    sim.push(np.array([3]))
    with pytest.raises(oracle_mod.OracleError) as e:
        sim.push(np.array([4]))
    assert e.value.code == oracle_mod.E_FULL                 # current + 1 future already buffered
    with pytest.raises(oracle_mod.OracleError) as e:
        sim.gather(np.array([3]))
    assert e.value.code == oracle_mod.E_ORDER                # not the head
    with pytest.raises(oracle_mod.OracleError) as e:
        sim.gather(np.array([1, 20]))
    assert e.value.code == oracle_mod.E_RANGE
    assert sim.batch == 0 and sim.window_count == 2          # failed calls leave the state alone
    sim.gather(np.array([2, 1, 1]))
    assert sim.batch == 1
    with pytest.raises(oracle_mod.OracleError):
        oracle_mod.Sim(20, 5, 2, 0)                          # lines not a multiple of ways
    with pytest.raises(oracle_mod.OracleError):
        oracle_mod.Sim(20, 4, 2, 0).push(np.array([1]))      # depth 0 takes no pushes


# -------------------------------------------------------------- sampler

def _tree(first_hop_degree):
    """node 0 -> 1..5; node i in 1..5 -> `first_hop_degree` leaves of its own."""
    indptr, indices, nxt = [0], [], 6
    indices += [1, 2, 3, 4, 5]
    indptr.append(len(indices))
    for _ in range(1, 6):
        indices += list(range(nxt, nxt + first_hop_degree))
        nxt += first_hop_degree
        indptr.append(len(indices))
    while len(indptr) < nxt + 1:
        indptr.append(len(indices))
    return nxt, np.array(indptr), np.array(indices)


def test_sampler_worked_example(oracle_mod):
    """Section 2.2.2: fanout 3, two layers, one target node: 1 + 3 + 6 = 10
    vertices and 9 edges when the first-hop nodes have two neighbours each
    ('up to three'), and at most 1 + 3 + 9."""
    n, indptr, indices = _tree(2)
    g = oracle_mod.Graph(0, n, csr=(indptr, indices))
    g13 = oracle_mod.Graph(0, *(_tree(4)[:1]), csr=_tree(4)[1:])
    # the single seed is hashed over all nodes: keep the minibatches whose seed is the tree's root
    hits = 0
    for batch in range(400):
        raw = g.sample(11, batch, [3, 3], 1)
        if raw[0] != 0:
            continue
        hits += 1
        assert len(set(raw.tolist())) == GOLDEN["sampling_example_vertices"]
        assert len(raw) - 1 == GOLDEN["sampling_example_edges"]
        first = raw[1:4].tolist()
        assert len(set(first)) == 3 and set(first) <= {1, 2, 3, 4, 5}
        for v in first:                                              # degree <= fanout: all neighbours
            assert set(indices[indptr[v]:indptr[v + 1]].tolist()) <= set(raw[4:].tolist())
        raw13 = g13.sample(11, batch, [3, 3], 1)
        if raw13[0] == 0:
            assert len(raw13) == 13 and len(set(raw13.tolist())) == 13   # the bound 1 + 3 + 9
    assert hits > 0


def test_sampler_is_uniform_without_replacement(oracle_mod):
    deg, f = 12, 5
    indptr = np.array([0, deg] + [deg] * deg)
    indices = np.arange(1, deg + 1)
    g = oracle_mod.Graph(0, deg + 1, csr=(indptr, indices))
    counts = np.zeros(deg + 1)
    pair = np.zeros((deg + 1, deg + 1))
    trials = 0
    for batch in range(60000):
        raw = g.sample(99, batch, [f], 1)
        if raw[0] != 0:
            continue
        trials += 1
        nb = raw[1:]
        assert len(nb) == f and len(set(nb.tolist())) == f          # distinct slots
        counts[nb] += 1
        pair[np.ix_(nb, nb)] += 1
    assert trials > 3000
    p = f / deg
    sigma = np.sqrt(trials * p * (1 - p))
    assert np.all(np.abs(counts[1:] - trials * p) < 5 * sigma)      # every slot equally likely
    p2 = f * (f - 1) / (deg * (deg - 1))                             # every pair equally likely
    off = pair[1:, 1:][~np.eye(deg, dtype=bool)]
    assert np.all(np.abs(off - trials * p2) < 5 * np.sqrt(trials * p2))


# ------------------------------------------------------------- Eq. 2-3

def test_overlapped_access_model(oracle_mod):
    """Section 3.2 Eq. 2-3 and the Section 4.2 example: Optane, 1.5 M IOPS at
    4 KB, 25 us initial + 5 us termination latency, 95 % of peak.  The paper
    prints 812 accesses; its text does not say which latency terms entered, and
    the formula with the stated 25 + 5 us gives 855 (5 % apart)."""
    iops, ti, tt, r = GOLDEN["optane_peak_iops"], GOLDEN["initial_latency_s"], GOLDEN["termination_latency_s"], 0.95
    n = oracle_mod.accum_threshold(iops, ti, tt, r, 1)
    assert abs(n - 855.0) < 1e-6
    assert abs(n - GOLDEN["optane_95pct_accesses"]) / GOLDEN["optane_95pct_accesses"] < 0.06
    # the defining fixed point: N = IOPS_achieved * (Ti + N / IOPS_peak + Tt)
    assert abs(n - r * iops * (ti + n / iops + tt)) < 1e-6
    # SSDs add up: twice the drives need twice the accesses in flight
    assert abs(oracle_mod.accum_threshold(iops, ti, tt, r, 2) - 2 * n) < 1e-6


def test_accumulator_groups_hand_traced(oracle_mod):
    """Section 3.2: iterations are merged until their node accesses pass the threshold.  A hand-traced run at
    threshold 10 (node access = raw list entry; pending = distinct IDs of the open group):
      list                    raw  distinct  nodes in group  closes?  pending after
      [1 2 3]                  3      3           3            no         3
      [4 5 6 6 6]              5      3           8            no         6
      [7]                      1      1           9            no         7
      [8 .. 18]               11     11          20            yes        0
      [1]                      1      1           1            no         1
      (flush)                                                  yes        0   (1 row was waiting)
      [2 2]                    2      1           2            no         1
      [3 .. 12]               10     10          12            yes        0
    """
    sim = oracle_mod.Sim(100, 16, 4, 0)
    sim.set_accum(10)
    lists = [[1, 2, 3], [4, 5, 6, 6, 6], [7], list(range(8, 19)), [1]]
    want = [(3, 0), (6, 0), (7, 0), (0, 1), (1, 0)]
    for raw, (pending, flushed) in zip(lists, want):
        sim.gather(raw)
        assert sim.accum_last == (pending, flushed, 10)
    assert sim.flush() == 1 and sim.flush() == 0
    sim.gather([2, 2])
    assert sim.accum_last == (1, 0, 10)
    sim.gather(list(range(3, 13)))
    assert sim.accum_last == (0, 1, 10)
    # a group never holds more than 32 minibatches, however high the threshold
    sim = oracle_mod.Sim(100, 16, 4, 0)
    sim.set_accum(10**9)
    flushed = []
    for t in range(70):
        sim.gather([t % 100])
        flushed.append(sim.accum_last[1])
    assert [t for t, f in enumerate(flushed) if f] == [31, 63]
    # without an accumulator every gather moves its own rows
    sim = oracle_mod.Sim(100, 16, 4, 0)
    sim.gather([1, 2])
    assert sim.accum_last == (0, 1, 0)


@pytest.mark.parametrize("window", [0, 3])
def test_accumulator_changes_no_result_and_loses_no_row(oracle_mod, window):
    """Merging is scheduling only: counters, classes, rows and tags are those of the run without it; every
    distinct ID of every minibatch is pending exactly until its group closes."""
    rng, feats, plain, hot = tiny_setup(oracle_mod, window=window)
    _, _, merged, _ = tiny_setup(oracle_mod, window=window)
    merged.set_accum(700)
    batches = [rng.integers(0, 400, size=int(rng.integers(1, 300))) for _ in range(40)]
    a = run_stream(plain, batches, window)
    open_rows, moved, pushed = 0, 0, 0
    for t, raw in enumerate(batches):
        while window and pushed < len(batches) and pushed <= t + window:
            merged.push(batches[pushed])
            pushed += 1
        u, rows, stats = merged.gather(raw)
        assert np.array_equal(u, a[t][0]) and np.array_equal(rows, a[t][1]) and np.array_equal(stats, a[t][2])
        pending, flushed, limit = merged.accum_last
        assert limit == 700
        open_rows += len(u)
        if flushed:
            moved, open_rows = moved + open_rows, 0
        assert pending == open_rows
    assert moved + merged.flush() == sum(len(r[0]) for r in a)
    assert np.array_equal(plain.tags, merged.tags) and np.array_equal(plain.stamps, merged.stamps)


def test_adaptive_accumulator_threshold_follows_the_redirected_share(oracle_mod):
    """Section 3.2, last paragraph: the threshold follows the accesses that are redirected to CPU / GPU
    memory.  With N store accesses wanted per launch, the node-access threshold is ceil(N * A / S) over the
    gathers at least 16 back (A node accesses, S store accesses), within [N, 8 N]."""
    LAG, N = 16, 50
    # (1) nothing is redirected and lists hold no repeats: every node access is a store access, threshold N
    sim = oracle_mod.Sim(10_000, 4, 4, 0)                       # a 4-line cache: practically everything misses
    sim.set_accum(N, 1)
    for t in range(60):
        sim.gather(np.arange(100 * t, 100 * t + 20))
        assert sim.accum_last[2] == N
    # (2) every ID listed twice: two node accesses per store access, threshold 2 N once counters 16 back exist
    sim = oracle_mod.Sim(10_000, 4, 4, 0)
    sim.set_accum(N, 1)
    for t in range(60):
        ids = np.arange(100 * t, 100 * t + 20)
        sim.gather(np.concatenate([ids, ids]))
        assert sim.accum_last[2] == (N if t <= LAG else 2 * N), t
    # (3) a quarter of the IDs pinned in the CPU buffer: 4 node accesses per 3 store accesses
    sim = oracle_mod.Sim(10_000, 4, 4, 0)
    sim.set_hot(np.arange(0, 10_000, 4))
    sim.set_accum(N, 1)
    for t in range(60):
        sim.gather(np.arange(100 * t, 100 * t + 40))
        assert sim.accum_last[2] == (N if t <= LAG else -(-N * 4 // 3)), t
    # (4) a cache that holds everything: store accesses stop, the share redirected tends to 1, bounded at 8 N;
    #     against the definition written out
    sim = oracle_mod.Sim(64, 64, 4, 0)
    sim.set_accum(N, 1)
    A, S, hist = 0, 0, []
    for t in range(200):
        raw = np.arange(64) if t % 2 else np.arange(0, 64, 2)
        _, _, stats = sim.gather(raw)
        hist.append((len(raw), int(stats[3])))
        A = sum(h[0] for h in hist[:max(0, t - LAG)])
        S = sum(h[1] for h in hist[:max(0, t - LAG)])
        want = N if A == 0 else (8 * N if S == 0 else min(8 * N, max(N, -(-N * A // S))))
        assert sim.accum_last[2] == want, t
    assert sim.accum_last[2] == 8 * N


def test_line_fills_happen_without_output_rows(oracle_mod):
    """A minibatch gathered for its counters only still fills the lines it
    installs: later hits on them must return the store's bytes."""
    rng, feats, sim, hot = tiny_setup(oracle_mod, n=200, lines=64, ways=4, window=0, n_hot=0)
    first = np.arange(0, 40)
    sim.gather(first, want_rows=False)                       # installs 40 lines, rows not requested
    uniq, rows, stats, cls = sim.gather(first, want_cls=True)
    assert stats[1] == 40 and np.all(cls == oracle_mod.CLS_HIT)
    assert rows.tobytes() == feats[first].tobytes()


# ------------------------------------------------------- random base policy

def test_random_policy_picks_uniformly_and_respects_the_window(oracle_mod):
    """Section 3.4's base policy: the victim is a random line; with window buffering lines whose
    node a buffered minibatch reuses are still never evicted, and empty ways are used first."""
    ways = 8
    counts = np.zeros(ways)
    trials = 0
    for seed in range(1500):
        sim = oracle_mod.Sim(1000, ways, ways, 0)           # one set
        sim.set_policy(1, seed)
        sim.gather(np.arange(ways), want_rows=False)         # fills the empty ways in way order
        assert sim.tags.tolist() == list(range(ways))
        sim.gather(np.array([500]), want_rows=False)         # one miss: which way goes?
        gone = [w for w in range(ways) if sim.tags[w] == 500]
        assert len(gone) == 1
        counts[gone[0]] += 1
        trials += 1
    p = 1.0 / ways
    assert np.all(np.abs(counts - trials * p) < 5 * np.sqrt(trials * p * (1 - p)))
    # pinned lines survive: nodes 0..3 are reused by the buffered next minibatch
    for seed in range(200):
        sim = oracle_mod.Sim(1000, ways, ways, 1)
        sim.set_policy(1, seed)
        b0, b1, b2 = np.arange(ways), np.array([600, 601, 602, 603]), np.array([0, 1, 2, 3])
        sim.push(b0); sim.push(b1)
        sim.gather(b0, want_rows=False)
        sim.push(b2)
        sim.gather(b1, want_rows=False)                      # four misses, only ways 4..7 are safe to evict
        assert sim.tags[:4].tolist() == [0, 1, 2, 3]
        assert sorted(sim.tags[4:].tolist()) == [600, 601, 602, 603]


def test_random_policy_against_an_independent_model(oracle_mod):
    """Depth 0, random policy: a Python model that orders occupied evictable ways by the documented hash."""
    n, n_sets, ways, seed = 400, 5, 4, 77
    sim = oracle_mod.Sim(n, n_sets * ways, ways, 0)
    sim.set_policy(1, seed)
    tags = [[-1] * ways for _ in range(n_sets)]
    rng = np.random.default_rng(8)
    for t, raw in enumerate(zipf_batches(rng, n, 40, 30, a=1.2)):
        ids = sorted(set(raw.tolist()))
        touched = [set() for _ in range(n_sets)]
        missing = {}
        hits = 0
        for v in ids:
            s = v % n_sets
            if v in tags[s]:
                hits += 1
                touched[s].add(tags[s].index(v))
            else:
                missing.setdefault(s, []).append(v)
        byp = 0
        for s, vs in missing.items():
            cand = [w for w in range(ways) if w not in touched[s]]
            def order(w):
                if tags[s][w] == -1:
                    return (-1, w)
                return (int(wl.hash_chain(seed, 8, t, s, w)) >> 9, w)
            cand.sort(key=order)
            for k, v in enumerate(vs):
                if k < len(cand):
                    tags[s][cand[k]] = v
                else:
                    byp += 1
        _, _, stats, _ = sim.gather(raw, want_cls=True)
        assert (stats[0], stats[1], stats[4]) == (len(ids), hits, byp)
        assert sim.tags.tolist() == [x for row in tags for x in row]


# -------------------------------------------------------- hot-node scores

def test_visit_scores_closed_form_and_against_sampling(oracle_mod):
    """Expected appearances per node: exact on a hand graph, and equal to the
    sampler's empirical hop-1 frequencies within sampling error."""
    one = float(1 << 32)
    # star: node 0 -> 1..6 (degree 6), every other node has no neighbours; 2 seeds, fanout 3
    indptr = np.array([0, 6, 6, 6, 6, 6, 6, 6])
    indices = np.arange(1, 7)
    g = oracle_mod.Graph(0, 7, csr=(indptr, indices))
    sc = g.visit_scores([3], 2) / one
    lam0 = 2 / 7
    assert abs(sc[0] - lam0) < 1e-6                                  # nobody points to node 0
    assert np.allclose(sc[1:], lam0 + lam0 * 3 / 6, atol=1e-6)       # seed mass + lam0 * min(6, 3) / 6 per slot
    # two hops on a chain 0 -> 1 -> 2: mass moves one node per hop, clamped presence <= 1
    g2 = oracle_mod.Graph(0, 3, csr=(np.array([0, 1, 2, 2]), np.array([1, 2])))
    sc2 = g2.visit_scores([5, 5], 6) / one                           # lam0 = 2 > 1: presence clamps to 1
    assert np.allclose(sc2, [2.0, 2.0 + 1.0, 2.0 + 1.0 + 1.0], atol=1e-6)
    # against the sampler itself (one hop, few seeds: no clamping, no dedup effects)
    cfg = CONFIGS["tiny"]
    gt = oracle_mod.Graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max)
    sc = gt.visit_scores([10], 32) / one
    cnt = np.zeros(cfg.n_nodes)
    n_b = 1500
    for b in range(n_b):
        cnt += np.bincount(gt.sample(5, b, [10], 32), minlength=cfg.n_nodes)
    top = np.argsort(-sc)[:40]
    sigma = np.sqrt(sc[top] / n_b)
    assert np.all(np.abs(cnt[top] / n_b - sc[top]) < 5 * sigma + 0.02 * sc[top])
    assert abs(cnt.sum() / n_b - sc.sum()) / sc.sum() < 0.03


def test_reverse_pagerank_against_closed_forms_and_a_linear_solve(oracle_mod):
    """Weighted reverse PageRank (Section 3.3): uniform on a ring, the geometric series on a chain (which also
    fixes the direction of the flow), the two-unknown closed form on a star, and the stationary solution of the
    linear system from numpy on a random multigraph."""
    total = float(1 << 44)
    d16, d = 55705, 55705 / 65536
    # ring v -> v+1: every node keeps 1/n
    n = 12
    ring = oracle_mod.Graph(0, n, csr=(np.arange(n + 1), (np.arange(n) + 1) % n))
    r = ring.reverse_pagerank(d16, 50) / total
    assert np.allclose(r, 1 / n, rtol=1e-9, atol=1e-11)
    # chain 0 -> 1 -> ... -> 7, node 7 keeps nothing: r(k) = t * (1 - d^(k+1)) / (1 - d), t = (1 - d) / n
    n = 8
    chain = oracle_mod.Graph(0, n, csr=(np.array(list(range(n)) + [n - 1]), np.arange(1, n)))
    r = chain.reverse_pagerank(d16, 40) / total
    want = (1 - d) / n * (1 - d ** np.arange(1, n + 1)) / (1 - d)
    assert np.allclose(r, want, rtol=1e-8, atol=1e-11)
    assert r[0] < r[1] < r[7]                                        # rank flows along the adjacency slots
    # star: hub 0 -> leaves 1..6, every leaf -> hub.  h = t + d*6*l, l = t + d*h/6
    n = 7
    indptr = np.array([0, 6, 7, 8, 9, 10, 11, 12])
    indices = np.array([1, 2, 3, 4, 5, 6, 0, 0, 0, 0, 0, 0])
    star = oracle_mod.Graph(0, n, csr=(indptr, indices))
    r = star.reverse_pagerank(d16, 400) / total
    t = (1 - d) / n
    h = t * (1 + 6 * d) / (1 - d * d)
    assert abs(r[0] - h) < 1e-9 and np.allclose(r[1:], t + d * h / 6, atol=1e-9)
    # random multigraph with repeated slots and self-loops: r = t * (I - d P^T)^-1 1, P[v, u] = slots(v -> u) / deg v
    rng = np.random.default_rng(3)
    n = 60
    deg = rng.integers(1, 9, n)
    indptr = np.concatenate([[0], np.cumsum(deg)])
    indices = rng.integers(0, n, indptr[-1])
    g = oracle_mod.Graph(0, n, csr=(indptr, indices))
    P = np.zeros((n, n))
    for v in range(n):
        for u in indices[indptr[v]:indptr[v + 1]]:
            P[v, u] += 1 / deg[v]
    want = np.linalg.solve(np.eye(n) - d * P.T, np.full(n, (1 - d) / n))
    r = g.reverse_pagerank(d16, 300) / total
    assert np.allclose(r, want, rtol=1e-7, atol=1e-10)
    assert abs(r.sum() - 1) < 1e-7                                   # no node without slots: mass is kept
    # a few iterations: equal to the same recurrence in float64
    x = np.full(n, 1 / n)
    for _ in range(3):
        x = (1 - d) / n + d * (P.T @ x)
    assert np.allclose(g.reverse_pagerank(d16, 3) / total, x, rtol=1e-7)
    # no damping mass: the uniform start stays
    assert len(set(g.reverse_pagerank(0, 5).tolist())) == 1


# ------------------------------------------------ several rows per cache line

def _drive(sim, lists, window, want_rows=False):
    """window protocol: keep window + 1 lists buffered; returns per-minibatch (unique, rows, stats, classes)"""
    res, pushed = [], 0
    for t, raw in enumerate(lists):
        while window and pushed < len(lists) and pushed <= t + window:
            sim.push(lists[pushed])
            pushed += 1
        res.append(sim.gather(raw, want_rows=want_rows, want_cls=True))
    return res


@pytest.mark.parametrize("P,window,policy", [(2, 0, None), (8, 3, None), (4, 2, (1, 77)), (8, 0, (1, 5)), (3, 4, None)])
def test_rows_per_line_reduces_to_one_row_per_line_over_line_numbers(oracle_mod, P, window, policy):
    """With P rows per line the cache works on store-line numbers b = id div P: its tags and stamps must be those
    of the (already pinned) one-row-per-line simulator fed the distinct line numbers of every list, and every
    requested row must have the class its line has there."""
    rng = np.random.default_rng(1000 + P)
    n, ways, n_sets = 1003, 4, 11                              # the last line of the table is partial
    lists = [np.minimum(rng.zipf(1.15, size=int(rng.integers(1, 400))) - 1, n - 1) for _ in range(40)]
    sim = oracle_mod.Sim(n, ways * n_sets, ways, window)
    sim.set_rows_per_line(P)
    ref = oracle_mod.Sim((n + P - 1) // P, ways * n_sets, ways, window)
    if policy:
        sim.set_policy(*policy)
        ref.set_policy(*policy)
    got = _drive(sim, lists, window)
    want = _drive(ref, [np.unique(np.asarray(l) // P) for l in lists], window)
    for t, ((u, _, stats, cls), (ub, _, _, clsb)) in enumerate(zip(got, want)):
        line_class = dict(zip(ub.tolist(), clsb.tolist()))
        expect = np.array([line_class[int(v) // P] for v in u])
        assert np.array_equal(cls, expect), t
        assert stats.tolist() == [len(u), int((expect == 0).sum()), 0, int((expect >= 2).sum()), int((expect == 3).sum())]
    assert np.array_equal(sim.tags, ref.tags) and np.array_equal(sim.stamps, ref.stamps)


def test_rows_per_line_brings_the_neighbours_in_and_moves_the_right_bytes(oracle_mod):
    rng = np.random.default_rng(8)
    n, R, P = 77, 48, 4                                         # 20 lines, the last holds one row
    store = rng.integers(0, 256, size=(n, R), dtype=np.uint8)
    sim = oracle_mod.Sim(n, 8, 2, 0, R, P * R + 16, store)
    sim.set_rows_per_line(P)
    u, rows, stats = sim.gather([5, 76])                        # lines 1 and 19 come in
    assert stats.tolist() == [2, 0, 0, 2, 0] and np.array_equal(rows, store[[5, 76]])
    u, rows, stats = sim.gather([4, 6, 7, 76, 9])               # rows 4, 6, 7 were never asked for: hits all the same
    assert stats.tolist() == [5, 4, 0, 1, 0] and np.array_equal(rows, store[[4, 6, 7, 9, 76]])
    # two rows of one missing line in one minibatch: two misses, one line
    u, rows, stats = sim.gather([40, 41, 43])
    assert stats.tolist() == [3, 0, 0, 3, 0] and sorted(t for t in sim.tags.tolist() if t >= 0) == [1, 2, 10, 19]
    # random traffic with a CPU buffer and a window: every gathered row is the store's row
    sim = oracle_mod.Sim(n, 8, 2, 2, R, P * R, store)
    sim.set_rows_per_line(P)
    sim.set_hot([3, 40, 41])
    lists = [rng.integers(0, n, size=int(rng.integers(1, 60))) for _ in range(30)]
    for (u, rows, stats, cls), raw in zip(_drive(sim, lists, 2, want_rows=True), lists):
        assert np.array_equal(u, np.unique(raw)) and np.array_equal(rows, store[u])
        assert stats[1] + stats[2] + stats[3] == stats[0]
        assert stats[2] == len(set(u.tolist()) & {3, 40, 41})
    # a cache with a line for every store line: one row of each line, then nothing misses any more
    sim = oracle_mod.Sim(n, 20, 4, 0)
    sim.set_rows_per_line(P)
    sim.gather(np.arange(0, n, P))
    u, _, stats = sim.gather(np.arange(n), want_rows=False)
    assert stats.tolist() == [n, n, 0, 0, 0]
    # the setting belongs before the first minibatch and must fit the line
    with pytest.raises(oracle_mod.OracleError):
        sim.set_rows_per_line(2)
    with pytest.raises(oracle_mod.OracleError):
        oracle_mod.Sim(n, 8, 2, 0, R, 2 * R, store).set_rows_per_line(3)


def test_rows_per_line_pins_a_line_while_any_of_its_rows_is_needed(oracle_mod):
    """One set of two ways, lines of two rows: line 0 is needed again two minibatches later through its *other*
    row, so the window keeps it and the plain LRU does not."""
    lists = [[0], [2], [4], [1]]                                # lines 0, 1, 2, then line 0 again via row 1
    for window, last in ((0, [1, 0, 0, 1, 0]), (3, [1, 1, 0, 0, 0])):
        sim = oracle_mod.Sim(64, 2, 2, window)
        sim.set_rows_per_line(2)
        res = _drive(sim, lists, window)
        assert res[3][2].tolist() == last, window
        if window:                                              # line 2 took the way of line 1, which nothing needs again
            assert res[2][2].tolist() == [1, 0, 0, 1, 0]


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """tests/oracle_sanitize.c drives the whole oracle through the Tiny configuration (three variants of the
    simulator) in a program built with -fsanitize=address,undefined; any report fails the run."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = tmp_path / "oracle_sanitize"
    build = subprocess.run(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-o", str(exe),
                            os.path.join(root, "tests", "oracle_sanitize.c"), "-lm"], capture_output=True, text=True)
    if build.returncode != 0 and "sanitize" in build.stderr:
        pytest.skip("this compiler has no sanitizer runtime")
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0")   # something else may be preloaded
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0 and "oracle sanitize ok" in run.stdout, run.stdout + run.stderr
