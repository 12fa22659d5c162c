"""The GPU neighbourhood sampler against the oracle's sampler: raw ID lists bit
for bit (length, order, duplicates), for uniform and Zipf-ranked seeds, both ID
widths, graph in GPU memory and zero-copy from pinned host memory; then the
whole sample -> push -> gather chain without the host ever seeing a list."""
import numpy as np
import pytest

import workload as wl
from workload import CONFIGS

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2306_16384_amd.session import GatherSession, GraphSampler
    return torch, GatherSession, GraphSampler


def sample_gpu(torch, gs, seed, batch, fanouts, n_seeds, rank_table=None, perm=(0, 0)):
    cap = gs.capacity(fanouts, n_seeds)
    raw = torch.full((max(cap, 1),), -5, dtype=gs.torch_id, device="cuda")
    n_raw = torch.zeros(1, dtype=torch.int32, device="cuda")
    gs.sample(seed, batch, fanouts, n_seeds, raw, n_raw, rank_table=rank_table, perm=perm)
    torch.cuda.synchronize()
    n = int(n_raw.item())
    assert bool((raw[n:] == -5).all())                      # nothing written past the reported length
    return raw[:n].cpu().numpy().astype(np.int64)


@pytest.mark.parametrize("name,n,dtype,zero_copy", [("tiny", None, np.int32, False), ("tiny", None, np.int64, True),
                                                    ("medium", 150_000, np.int64, False), ("large", 300_000, np.int64, False)])
def test_raw_lists_equal_the_oracle_sampler(env, oracle_mod, name, n, dtype, zero_copy):
    torch, _, GraphSampler = env
    cfg = CONFIGS[name]
    n = n or cfg.n_nodes
    d_max = min(n - 1, 65535)
    g = oracle_mod.Graph(cfg.seed, n, cfg.ell, cfg.p4, d_max)
    print(f"[sampler {name}] n={n} E={g.n_edges} ids={np.dtype(dtype).name} zero_copy={zero_copy}", flush=True)
    with GraphSampler(g.indptr, g.indices.astype(dtype), zero_copy=zero_copy) as gs:
        for batch in (0, 1, 5, 1000):
            want = g.sample(cfg.seed, batch, cfg.fanouts, cfg.n_seeds)
            got = sample_gpu(torch, gs, cfg.seed, batch, cfg.fanouts, cfg.n_seeds)
            np.testing.assert_array_equal(got, want, err_msg=f"{name} batch {batch}")
        # other shapes: one layer, deep and narrow, fanout above every degree, a single seed, no layer at all
        for fanouts, n_seeds in (((3,), 17), ((2, 2, 2, 2, 2), 9), ((64, 64), 5), ((7, 3), 1), ((), 33)):
            want = g.sample(cfg.seed + 1, 2, fanouts, n_seeds)
            got = sample_gpu(torch, gs, cfg.seed + 1, 2, fanouts, n_seeds)
            np.testing.assert_array_equal(got, want, err_msg=f"{name} fanouts {fanouts}")


def test_zipf_ranked_seeds(env, oracle_mod):
    torch, _, GraphSampler = env
    cfg = CONFIGS["medium"]
    n = 80_000
    g = oracle_mod.Graph(cfg.seed, n, cfg.ell, cfg.p4, min(n - 1, 65535))
    with GraphSampler(g.indptr, g.indices) as gs:
        for s_exp in (0.0, 0.8, 1.2):
            tab = wl.synth.zipf_rank_table(n, s_exp)
            perm = wl.synth.perm_params(cfg.seed, n)
            tab_dev = torch.from_numpy(tab.view(np.int64)).cuda()
            for batch in (0, 4):
                want = g.sample(cfg.seed, batch, (25, 10), 512, rank_table=tab, perm=perm)
                got = sample_gpu(torch, gs, cfg.seed, batch, (25, 10), 512, rank_table=tab_dev, perm=perm)
                np.testing.assert_array_equal(got, want)


def test_hand_built_tree_matches_the_worked_example(env, oracle_mod):
    """Fanout 3, two layers, one target: 1 + 3 + 6 vertices when first-hop nodes have two neighbours."""
    torch, _, GraphSampler = env
    indptr, indices, nxt = [0], [1, 2, 3, 4, 5], 6
    indptr.append(5)
    for _ in range(5):
        indices += [nxt, nxt + 1]
        nxt += 2
        indptr.append(len(indices))
    while len(indptr) < nxt + 1:
        indptr.append(len(indices))
    g = oracle_mod.Graph(0, nxt, csr=(np.array(indptr), np.array(indices)))
    with GraphSampler(np.array(indptr), np.array(indices, dtype=np.int64)) as gs:
        seen = 0
        for batch in range(200):
            want = g.sample(11, batch, [3, 3], 1)
            got = sample_gpu(torch, gs, 11, batch, [3, 3], 1)
            np.testing.assert_array_equal(got, want)
            if got[0] == 0:
                seen += 1
                assert len(got) == 10 and len(set(got.tolist())) == 10
        assert seen > 0


def test_sample_push_gather_without_the_host(env, oracle_mod):
    """Lists go sampler -> window -> gather entirely on the device; results equal
    the oracle fed with its own sampler's lists."""
    torch, GatherSession, GraphSampler = env
    cfg = CONFIGS["tiny"]
    g = oracle_mod.Graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max)
    table = wl.normal_table(np.float32)
    feats = oracle_mod.feat_rows(cfg.seed, np.arange(cfg.n_nodes), cfg.dim, table).view(np.uint8).reshape(cfg.n_nodes, -1)
    hot = g.hot_nodes(cfg.cpu_rows)
    n_b, W = 16, cfg.window
    lists = [g.sample(cfg.seed, b, cfg.fanouts, cfg.n_seeds) for b in range(n_b)]
    sim = oracle_mod.Sim(cfg.n_nodes, cfg.cache_lines, cfg.ways, W, cfg.row_bytes, cfg.line_bytes, feats)
    sim.set_hot(hot)
    want, pushed = [], 0
    for t in range(n_b):
        while pushed < n_b and pushed <= t + W:
            sim.push(lists[pushed])
            pushed += 1
        want.append(sim.gather(lists[t]))
    with GraphSampler(g.indptr, g.indices.astype(np.int32)) as gs, \
            GatherSession(cfg.n_nodes, cfg.row_bytes, np.int32, cfg.cache_lines, cfg.ways, cfg.line_bytes, W) as ses:
        ses.store_view()[:] = feats
        ses.pin_hot(hot)
        cap = gs.capacity(cfg.fanouts, cfg.n_seeds)
        ses.reserve(cap)
        bufs = [(torch.empty(cap, dtype=torch.int32, device="cuda"), torch.zeros(1, dtype=torch.int32, device="cuda"))
                for _ in range(n_b)]
        outs, uqs, seqs, pushed = [], [], [], 0
        for t in range(n_b):
            while pushed < n_b and pushed <= t + W:
                raw, n_raw = bufs[pushed]
                gs.sample(cfg.seed, pushed, cfg.fanouts, cfg.n_seeds, raw, n_raw)
                ses.push_dev(raw, n_raw)
                pushed += 1
            out = torch.zeros((cap, cfg.row_bytes), dtype=torch.uint8, device="cuda")
            uq = torch.zeros(cap, dtype=torch.int32, device="cuda")
            seqs.append(ses.gather(None, out, uq))
            outs.append(out); uqs.append(uq)
        torch.cuda.synchronize()
        for t in range(n_b):
            u, rows, stats = want[t]
            st = ses.stats(seqs[t])
            assert st.as_tuple() == tuple(int(x) for x in stats), (t, st.as_tuple(), stats.tolist())
            assert np.array_equal(uqs[t][:len(u)].cpu().numpy(), u.astype(np.int32))
            assert np.array_equal(outs[t][:len(u)].cpu().numpy(), rows)


@pytest.mark.parametrize("name,n,dtype", [("tiny", None, np.int32), ("medium", 200_000, np.int64), ("large", 250_000, np.int64)])
def test_visit_scores_equal_the_oracle(env, oracle_mod, name, n, dtype):
    torch, _, GraphSampler = env
    cfg = CONFIGS[name]
    n = n or cfg.n_nodes
    g = oracle_mod.Graph(cfg.seed, n, cfg.ell, cfg.p4, min(n - 1, 65535))
    with GraphSampler(g.indptr, g.indices.astype(dtype)) as gs:
        for fanouts, n_seeds in ((cfg.fanouts, cfg.n_seeds), ((64,), 3), ((), 10), ((1, 1, 1, 1), 100_000)):
            want = g.visit_scores(fanouts, n_seeds)
            got = gs.visit_scores(fanouts, n_seeds).cpu().numpy().view(np.uint64)
            np.testing.assert_array_equal(got, want, err_msg=f"{name} {fanouts}")


@pytest.mark.parametrize("name,n,dtype", [("tiny", None, np.int32), ("medium", 200_000, np.int64), ("large", 250_000, np.int64)])
def test_reverse_pagerank_equals_the_oracle(env, oracle_mod, name, n, dtype):
    """Section 3.3's hot-node metric: integer power iteration, bit for bit, odd and even iteration counts."""
    torch, _, GraphSampler = env
    cfg = CONFIGS[name]
    n = n or cfg.n_nodes
    g = oracle_mod.Graph(cfg.seed, n, cfg.ell, cfg.p4, min(n - 1, 65535))
    with GraphSampler(g.indptr, g.indices.astype(dtype)) as gs:
        for d16, iters in ((55705, 0), (55705, 1), (55705, 6), (32768, 3), (65536, 2), (0, 2)):
            want = g.reverse_pagerank(d16, iters)
            got = gs.reverse_pagerank(d16, iters).cpu().numpy().view(np.uint64)
            np.testing.assert_array_equal(got, want, err_msg=f"{name} d16={d16} iters={iters}")


def test_reverse_pagerank_on_a_graph_with_empty_adjacency_lists(env, oracle_mod):
    torch, _, GraphSampler = env
    rng = np.random.default_rng(11)
    n = 5000
    deg = rng.integers(0, 6, n)                                       # a fifth of the nodes has no slots
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    indices = rng.integers(0, n, indptr[-1]).astype(np.int64)
    g = oracle_mod.Graph(0, n, csr=(indptr, indices))
    with GraphSampler(indptr, indices) as gs:
        want = g.reverse_pagerank(55705, 9)
        got = gs.reverse_pagerank(55705, 9).cpu().numpy().view(np.uint64)
        np.testing.assert_array_equal(got, want)
    with pytest.raises(Exception):
        with GraphSampler(indptr, indices) as gs:
            gs.reverse_pagerank(70000, 3)
