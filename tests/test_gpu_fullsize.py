"""Parity at the benchmark's sizes and launch configuration: Medium at full
size (every counter of every minibatch, full tensors on a subset); Large and
the skew configuration at the node count the benchmark runs, and the
cache-resident configuration at its full size (counters of every minibatch,
distinct-ID lists exact, sampled rows of every class against the oracle's
closed-form feature rows, final tags and stamps)."""
import numpy as np
import pytest

import workload as wl
from workload import CONFIGS

pytestmark = pytest.mark.gpu

# GIDS_FULL_PARITY=1 runs every minibatch the configurations name (500 / 300 / 1000; several minutes of host
# time for sampling and the oracle); the default runs a prefix of each.
import os
EVERY = os.environ.get("GIDS_FULL_PARITY", "0") == "1"


def drive(ses, torch, raws, window, cap_rows, row_bytes, keep):
    """Benchmark protocol: keep window + 1 lists buffered, gather the head list."""
    dev = [ses.to_device(r) for r in raws]
    ses.reserve(max(len(r) for r in raws))
    outs, uniqs, seqs, pushed = {}, {}, [], 0
    stats = {}                                                # the library keeps the counters of the last 64 gathers
    scratch = [torch.empty((cap_rows, row_bytes), dtype=torch.uint8, device="cuda") for _ in range(2)]
    uq_scratch = torch.empty(cap_rows, dtype=ses.torch_id, device="cuda")
    for t in range(len(raws)):
        while window and pushed < len(raws) and pushed <= t + window:
            ses.push(dev[pushed])
            pushed += 1
        if t in keep:
            outs[t] = torch.empty((cap_rows, row_bytes), dtype=torch.uint8, device="cuda")
            uniqs[t] = torch.empty(cap_rows, dtype=ses.torch_id, device="cuda")
            seqs.append(ses.gather(None if window else dev[t], outs[t], uniqs[t]))
        else:
            seqs.append(ses.gather(None if window else dev[t], scratch[t & 1], uq_scratch))
        if t >= 40:
            stats[t - 40] = ses.stats(seqs[t - 40])
    torch.cuda.synchronize()
    for t in range(max(0, len(raws) - 40), len(raws)):
        stats[t] = ses.stats(seqs[t])
    return outs, uniqs, stats


def test_medium_full_size(oracle_mod):
    import torch
    from paper_2306_16384_amd.session import GatherSession
    cfg = CONFIGS["medium"]
    n_b = cfg.n_batches                                       # all 200 minibatches of the configuration
    print(f"[fullsize medium] N={cfg.n_nodes} batches={n_b}", flush=True)
    g = wl.make_graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max, native=True)
    table = wl.normal_table(np.float16)
    hot = wl.hot_nodes(g, cfg.cpu_rows)
    raws = [wl.sample_minibatch(g, cfg.seed, b, cfg.fanouts, cfg.n_seeds) for b in range(n_b)]
    cap = max(len(np.unique(r)) for r in raws)
    keep = {0, 1, 9, 10, 23, 97, 150, n_b - 1}
    with GatherSession(cfg.n_nodes, cfg.row_bytes, np.int64, cfg.cache_lines, cfg.ways, cfg.line_bytes,
                       cfg.window) as ses:
        wl.fill_store(cfg.seed, cfg.n_nodes, cfg.dim, table, ses.store_address())
        ses.pin_hot(hot)
        outs, uniqs, stats_of = drive(ses, torch, raws, cfg.window, cap, cfg.row_bytes, keep)
        sim = oracle_mod.Sim(cfg.n_nodes, cfg.cache_lines, cfg.ways, cfg.window, cfg.row_bytes, cfg.line_bytes,
                             ses.store_view())
        sim.set_hot(hot)
        pushed = 0
        for t, raw in enumerate(raws):
            while pushed < n_b and pushed <= t + cfg.window:
                sim.push(raws[pushed])
                pushed += 1
            u, rows, stats = sim.gather(raw, want_rows=t in keep)
            st = stats_of[t]
            assert st.as_tuple() == tuple(int(x) for x in stats), (t, st.as_tuple(), stats.tolist())
            if t in keep:
                assert np.array_equal(uniqs[t][:len(u)].cpu().numpy(), u)
                assert np.array_equal(outs[t][:len(u)].cpu().numpy(), rows), f"minibatch {t}"
        tags, stamps = ses.snapshot()
        assert np.array_equal(tags, sim.tags) and np.array_equal(stamps, sim.stamps)


def pinnable(cfg_name, sizes):
    """The configuration at the first of `sizes` whose store this box can pin."""
    import paper_2306_16384_amd as gids
    for n_nodes in sizes:
        cfg = CONFIGS[cfg_name] if n_nodes == CONFIGS[cfg_name].n_nodes else wl.scaled(CONFIGS[cfg_name], n_nodes)
        try:
            probe = gids.gids_store_create(cfg.n_nodes, cfg.row_bytes, 8)
        except gids.GidsError as e:
            if e.code != gids.GIDS_E_NOMEM:
                raise
            print(f"[fullsize {cfg_name}] cannot pin {cfg.n_nodes * cfg.row_bytes / 1e9:.1f} GB, trying smaller", flush=True)
            continue
        gids.gids_store_destroy(probe)
        return cfg
    pytest.fail(f"cannot pin even {sizes[-1]} rows of host memory")


def sample_lists(g, cfg, n_b, rank_table=None):
    raws = []
    for b in range(n_b):
        raws.append(wl.sample_minibatch(g, cfg.seed, b, cfg.fanouts, cfg.n_seeds, rank_table))
        if b % 100 == 99:
            print(f"[fullsize {cfg.name}] sampled {b + 1} of {n_b} lists", flush=True)
    return raws


def run_big(oracle_mod, cfg, raws, keep, table, hot=None, after_each=None):
    """Counters of every minibatch, distinct-ID lists exact, rows of every class sampled against the oracle's
    closed-form feature rows, final tags and stamps."""
    import torch
    from paper_2306_16384_amd.session import GatherSession
    n_b = len(raws)
    cap = max(len(r) for r in raws)                           # raw length bounds the distinct count
    with GatherSession(cfg.n_nodes, cfg.row_bytes, np.int64, cfg.cache_lines, cfg.ways, cfg.line_bytes,
                       cfg.window) as ses:
        wl.fill_store(cfg.seed, cfg.n_nodes, cfg.dim, table, ses.store_address())
        if hot is not None:
            ses.pin_hot(hot)
        outs, uniqs, stats_of = drive(ses, torch, raws, cfg.window, cap, cfg.row_bytes, keep)
        sim = oracle_mod.Sim(cfg.n_nodes, cfg.cache_lines, cfg.ways, cfg.window)      # counts only
        if hot is not None:
            sim.set_hot(hot)
        rng = np.random.default_rng(0)
        pushed = 0
        for t, raw in enumerate(raws):
            while cfg.window and pushed < n_b and pushed <= t + cfg.window:
                sim.push(raws[pushed])
                pushed += 1
            u, _, stats, cls = sim.gather(raw, want_rows=False, want_cls=True)
            if t % 50 == 49:
                print(f"[fullsize {cfg.name}] oracle at minibatch {t + 1} of {n_b}", flush=True)
            st = stats_of[t]
            assert st.as_tuple() == tuple(int(x) for x in stats), (t, st.as_tuple(), stats.tolist())
            if after_each:
                after_each(t, st)
            if t in keep:
                assert np.array_equal(uniqs[t][:len(u)].cpu().numpy(), u)
                pick = []
                for k in range(4):                                # hit, CPU buffer, installed miss, bypass
                    idx = np.flatnonzero(cls == k)
                    if len(idx):
                        pick.append(rng.choice(idx, size=min(48, len(idx)), replace=False))
                pick = np.sort(np.concatenate(pick))
                got = outs[t][torch.from_numpy(pick).cuda()].cpu().numpy()
                want = oracle_mod.feat_rows(cfg.seed, u[pick], cfg.dim, table).view(np.uint8).reshape(len(pick), -1)
                assert np.array_equal(got, want), f"minibatch {t}"
        tags, stamps = ses.snapshot()
        assert np.array_equal(tags, sim.tags) and np.array_equal(stamps, sim.stamps)


def test_large_at_benchmark_size(oracle_mod):
    # the benchmark's node count; a box that pins less host memory runs the same test at half the size
    cfg = pinnable("large", (28_000_000, 14_000_000, 7_000_000))
    n_b = CONFIGS["large"].n_batches if EVERY else 150
    print(f"[fullsize large] N={cfg.n_nodes} lines={cfg.cache_lines} cpu_rows={cfg.cpu_rows} batches={n_b}", flush=True)
    g = wl.make_graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max, native=True)
    hot = wl.hot_nodes(g, cfg.cpu_rows)
    raws = sample_lists(g, cfg, n_b)
    run_big(oracle_mod, cfg, raws, {0, 9, 33, n_b - 1}, wl.normal_table(np.float16), hot=hot)


def test_skew_at_benchmark_size(oracle_mod):
    """The skew configuration (16 ways, Zipf-ranked seeds, depth 4) at the node count the benchmark runs."""
    cfg = pinnable("skew", (28_000_000, 14_000_000, 7_000_000))
    n_b = CONFIGS["skew"].n_batches if EVERY else 100
    print(f"[fullsize skew] N={cfg.n_nodes} lines={cfg.cache_lines} ways={cfg.ways} batches={n_b}", flush=True)
    g = wl.make_graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max, native=True)
    hot = wl.hot_nodes(g, cfg.cpu_rows)
    rank_table = wl.synth.zipf_rank_table(cfg.n_nodes, cfg.seed_zipf_s)
    raws = sample_lists(g, cfg, n_b, rank_table)
    run_big(oracle_mod, cfg, raws, {0, 5, n_b - 1}, wl.normal_table(np.float16), hot=hot)


def test_cache_resident_full_size(oracle_mod):
    """The cache-resident configuration at its full size (10 M rows of 3 KiB in 4 KiB lines, a cache that holds
    the whole table): lists that touch every row once, then sampled minibatches, which must all hit."""
    cfg = pinnable("resident", (10_000_000,))
    n_b = 200 if EVERY else 40                                # (the configuration names 1000: 19 GB of ID lists)
    print(f"[fullsize resident] N={cfg.n_nodes} lines={cfg.cache_lines} ways={cfg.ways} batches=10+{n_b}", flush=True)
    g = wl.make_graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max, native=True)
    step = 1_000_000
    raws = [np.arange(b, min(cfg.n_nodes, b + step), dtype=np.int64) for b in range(0, cfg.n_nodes, step)]
    n_pre = len(raws)
    raws += sample_lists(g, cfg, n_b)

    def all_hits_after_coverage(t, st):
        if t >= n_pre:
            assert st.n_miss == 0 and st.n_hit == st.n_unique, (t, st.as_tuple())
        else:
            assert st.n_miss == st.n_unique and st.n_bypass == 0, (t, st.as_tuple())

    run_big(oracle_mod, cfg, raws, {0, n_pre - 1, n_pre, n_pre + n_b - 1}, wl.normal_table(np.float32),
            after_each=all_hits_after_coverage)
