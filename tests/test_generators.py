"""The synthetic-input generators: the oracle's own C implementation against
the vectorised one in workload/, and both against what the definitions fix
(closed-form tail law, mean degree, in-degree proportional to out-degree, the
published first output of the mixing function's reference generator)."""
import numpy as np
import pytest

import workload as wl
from workload import CONFIGS

pytestmark = pytest.mark.filterwarnings("ignore::RuntimeWarning")


def test_mix64_published_vector(oracle_mod):
    # The mixer is the output function of the SplitMix64 generator; its first
    # output from state 0 is the widely published 0xE220A8397B1DCDAF.
    z = 0x9E3779B97F4A7C15
    assert oracle_mod.mix64(z) == 0xE220A8397B1DCDAF
    assert int(wl.mix64(z)) == 0xE220A8397B1DCDAF


def _both_graphs(oracle_mod, cfg, n=None):
    n = n or cfg.n_nodes
    d_max = min(n - 1, 65535)
    g_np = wl.make_graph(cfg.seed, n, cfg.ell, cfg.p4, d_max)
    g_c = oracle_mod.Graph(cfg.seed, n, cfg.ell, cfg.p4, d_max)
    return g_np, g_c


@pytest.mark.parametrize("name,n", [("tiny", None), ("medium", 60_000), ("large", 80_000)])
def test_graph_generators_agree(oracle_mod, name, n):
    cfg = CONFIGS[name]
    g_np, g_c = _both_graphs(oracle_mod, cfg, n)
    assert g_np.n_edges == g_c.n_edges
    np.testing.assert_array_equal(g_np.indptr, g_c.indptr)
    np.testing.assert_array_equal(g_np.indices, g_c.indices)
    k = max(1, g_np.n // 50)
    np.testing.assert_array_equal(wl.hot_nodes(g_np, k), g_c.hot_nodes(k))


@pytest.mark.parametrize("name", ["tiny", "medium"])
def test_degree_law(name):
    cfg = CONFIGS[name]
    deg = wl.synth.degrees_for(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max)
    assert deg.min() >= 1 and deg.max() <= cfg.d_max
    assert abs(deg.mean() - cfg.mean_degree) / cfg.mean_degree < 0.01
    # bounded Pareto: P(deg >= d) = P(ell / x^(p4/4) >= d) = (ell / d)^(4/p4) for 1 < d <= d_max
    for d in (2, 5, 20, 100):
        want = (cfg.ell / d) ** (4.0 / cfg.p4)
        got = (deg >= d).mean()
        sigma = np.sqrt(want * (1 - want) / cfg.n_nodes)
        assert abs(got - want) < 5 * sigma + 1e-4, (d, got, want)


def test_indegree_follows_outdegree():
    cfg = CONFIGS["medium"]
    n = 200_000
    g = wl.make_graph(cfg.seed, n, cfg.ell, cfg.p4, min(n - 1, 65535))
    deg = g.degrees()
    indeg = np.bincount(g.indices, minlength=n)
    hubs = np.argsort(-deg)[:50]
    # each edge slot lands on u with probability deg(u)/E  =>  indeg(u) ~ Binomial(E, deg(u)/E)
    for u in hubs:
        mu = float(deg[u])
        assert abs(indeg[u] - mu) < 6 * np.sqrt(mu) + 3
    assert indeg.sum() == g.n_edges
    assert g.indices.min() >= 0 and g.indices.max() < n


@pytest.mark.parametrize("name", ["tiny", "medium"])
def test_samplers_agree(oracle_mod, name):
    cfg = CONFIGS[name]
    n = min(cfg.n_nodes, 100_000)
    g_np, g_c = _both_graphs(oracle_mod, cfg, n)
    for b in (0, 1, 7):
        raw_np = wl.sample_minibatch(g_np, cfg.seed, b, cfg.fanouts, cfg.n_seeds)
        raw_c = g_c.sample(cfg.seed, b, cfg.fanouts, cfg.n_seeds)
        np.testing.assert_array_equal(raw_np, raw_c)


@pytest.mark.parametrize("dtype,dim", [(np.float32, 128), (np.float16, 1024)])
def test_features_agree_and_are_normal(oracle_mod, dtype, dim):
    table = wl.normal_table(dtype)
    ids = np.array([0, 1, 2, 12345, 999_999, 49_999_999], dtype=np.int64)
    a = wl.feature_rows(77, ids, dim, table)
    b = oracle_mod.feat_rows(77, ids, dim, table)
    np.testing.assert_array_equal(a.view(np.uint8), b.view(np.uint8))
    # native filler writes the same bytes
    out = np.empty((64, dim), dtype=dtype)
    wl.fill_store(77, 64, dim, table, out, row_lo=12300, native=True, threads=3)
    ref = oracle_mod.feat_rows(77, np.arange(12300, 12364), dim, table)
    np.testing.assert_array_equal(out.view(np.uint8), ref.view(np.uint8))
    # N(0,1): the table is the quantile function on a uniform grid
    big = wl.feature_rows(77, np.arange(2000), dim, table).astype(np.float64)
    assert abs(big.mean()) < 0.01 and abs(big.std() - 1.0) < 0.01
    assert abs(np.mean(np.abs(big) < 1.0) - 0.6827) < 0.005


def test_zipf_seed_draw_is_skewed():
    n = 100_000
    tab = wl.synth.zipf_rank_table(n, 1.2)
    seeds = np.concatenate([wl.minibatch_seeds(5, n, b, 2048, tab) for b in range(20)])
    assert seeds.min() >= 0 and seeds.max() < n
    _, counts = np.unique(seeds, return_counts=True)
    # rank 1 holds 1/zeta_n(1.2) of the mass (~0.2 for n = 1e5)
    w = np.arange(1, n + 1, dtype=np.float64) ** -1.2
    assert abs(counts.max() / len(seeds) - w[0] / w.sum()) < 0.02
    uni = np.concatenate([wl.minibatch_seeds(5, n, b, 2048, wl.synth.zipf_rank_table(n, 0.0)) for b in range(20)])
    assert np.unique(uni).size > 0.8 * uni.size


def test_skewed_seed_samplers_agree(oracle_mod):
    cfg = CONFIGS["medium"]
    n = 50_000
    g_np, g_c = _both_graphs(oracle_mod, cfg, n)
    for s_exp in (0.0, 0.8, 1.2):
        tab = wl.synth.zipf_rank_table(n, s_exp)
        perm = wl.synth.perm_params(cfg.seed, n)
        for b in (0, 3):
            raw_np = wl.sample_minibatch(g_np, cfg.seed, b, (25, 10), 512, tab)
            raw_c = g_c.sample(cfg.seed, b, (25, 10), 512, rank_table=tab, perm=perm)
            np.testing.assert_array_equal(raw_np, raw_c)


def test_layerwise_minibatch_has_fixed_layers_drawn_by_connection_count():
    """The layer-wise stream (Section 4.7's second sampler shape): every layer holds exactly its size of
    distinct nodes, all of them neighbours of the previous layer, and a node is kept with a probability that
    grows with the number of slots pointing to it."""
    cfg = CONFIGS["tiny"]
    g = wl.make_graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max, np.dtype(np.int32))
    sizes = (100, 150)
    n_seeds = 64
    for b in range(5):
        raw = wl.layerwise_minibatch(g, cfg.seed, b, sizes, n_seeds)
        assert np.array_equal(raw, wl.layerwise_minibatch(g, cfg.seed, b, sizes, n_seeds))
        assert len(raw) == n_seeds + sum(sizes)
        seeds, l1, l2 = raw[:n_seeds], raw[n_seeds:n_seeds + sizes[0]], raw[n_seeds + sizes[0]:]
        assert len(np.unique(l1)) == sizes[0] and len(np.unique(l2)) == sizes[1]
        for prev, layer in ((np.unique(seeds), l1), (l1, l2)):
            nb = np.concatenate([g.indices[g.indptr[v]:g.indptr[v + 1]] for v in prev])
            assert np.isin(layer, nb).all()
    # a layer larger than the neighbourhood keeps all of it
    raw = wl.layerwise_minibatch(g, cfg.seed, 0, (10**6,), n_seeds)
    nb = np.concatenate([g.indices[g.indptr[v]:g.indptr[v + 1]] for v in np.unique(raw[:n_seeds])])
    assert np.array_equal(raw[n_seeds:], np.unique(nb))
    # one layer from a fixed seed set, many minibatch counters: frequency rises with multiplicity
    hub = np.argsort(-(g.indptr[1:] - g.indptr[:-1]))[:20]
    nb = np.concatenate([g.indices[g.indptr[v]:g.indptr[v + 1]] for v in hub])
    ids, mult = np.unique(nb, return_counts=True)
    kept = np.zeros(cfg.n_nodes)
    import workload.synth as S
    orig = S.minibatch_seeds
    S.minibatch_seeds = lambda seed, n, batch, n_seeds, rank_table=None: hub.astype(np.int64)
    try:
        for b in range(300):
            raw = S.layerwise_minibatch(g, cfg.seed, b, (len(ids) // 4,), len(hub))
            kept[raw[len(hub):]] += 1
    finally:
        S.minibatch_seeds = orig
    # the definition, slot by slot, where the generator takes its short cut (few kept out of many slots)
    S.minibatch_seeds = lambda seed, n, batch, n_seeds, rank_table=None: hub.astype(np.int64)
    try:
        raw = S.layerwise_minibatch(g, cfg.seed, 7, (16,), len(hub))
    finally:
        S.minibatch_seeds = orig
    best = {}
    for v in np.unique(hub):
        for e in range(g.indptr[v], g.indptr[v + 1]):
            k = int(wl.hash_chain(cfg.seed, 9, 7, 0, e))
            u = int(g.indices[e])
            best[u] = min(best.get(u, 1 << 64), k)
    assert len(nb) > 4 * 16 + 1024
    want = sorted(sorted(best, key=lambda u: (best[u], u))[:16])
    assert raw[len(hub):].tolist() == want
    rate = kept[ids] / 300
    lo, hi = rate[mult == 1].mean(), rate[mult >= 3].mean()
    assert hi > lo + 0.2, (lo, hi)
    # weight-proportional race: P(keep) for multiplicity 1 is below the uniform share, above it for >= 3
    assert lo < 0.25 < hi


def test_frozen_degree_scale_is_what_the_bisection_gives():
    """workload/configs.py freezes `ell`; workload/calibrate.py is the script that solves it."""
    from workload import calibrate
    for name in ("tiny", "medium"):
        cfg = CONFIGS[name]
        assert abs(calibrate.solve(name) - cfg.ell) < 1e-9 * cfg.ell
