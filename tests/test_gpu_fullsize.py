"""Parity at the benchmark's sizes and launch configuration.

Medium at full size: counters and the whole tensor of all 200 minibatches
against the oracle.  Large, the nine points of the skew sweep (at the node
count the benchmark runs) and the cache-resident configuration (at its full
size): counters of every minibatch against the oracle's simulator, and on the
kept minibatches (the first window + 2, every 25th, the last) the distinct-ID
list exactly and EVERY gathered row against the plain definition
out[j] == store[unique[j]], the store itself being pinned to the oracle's
closed-form feature rows on a sample; final tags and stamps of every line.
The skew sweep runs a second time with a cache a few minibatches large, where
lines are evicted inside the run and the hit ratio moves with the window depth.
"""
import json
import os
import time

import numpy as np
import pytest

import workload as wl
from workload import CONFIGS

pytestmark = pytest.mark.gpu

# Medium, Large and the skew sweep run every minibatch their configurations name (200 / 500 / 300 per point).
# The cache-resident configuration names 1000 minibatches of 2.4 M raw IDs (19 GB of lists, minutes of host-side
# sampling): the default runs 40 after the covering lists, GIDS_FULL_PARITY=1 runs 200.
EVERY = os.environ.get("GIDS_FULL_PARITY", "0") == "1"


def kept_minibatches(n_b, window, first=0):
    """The subset whose whole tensors are compared: the first window + 2, every 25th, the last."""
    keep = set(range(first, min(n_b, first + window + 2))) | set(range(first, n_b, 25)) | {n_b - 1}
    return keep


def drive(ses, torch, raws, window, cap_rows, row_bytes, keep):
    """Benchmark protocol: keep window + 1 lists buffered, gather the head list (pushes on a stream of their
    own, as bench.py issues them)."""
    dev = [ses.to_device(r) for r in raws]
    ses.reserve(max(len(r) for r in raws))
    outs, uniqs, seqs, pushed = {}, {}, [], 0
    stats = {}                                                # the library keeps the counters of the last 64 gathers
    scratch = [torch.empty((cap_rows, row_bytes), dtype=torch.uint8, device="cuda") for _ in range(2)]
    uq_scratch = torch.empty(cap_rows, dtype=ses.torch_id, device="cuda")
    push_stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    for t in range(len(raws)):
        while window and pushed < len(raws) and pushed <= t + window:
            ses.push(dev[pushed], stream=push_stream)
            pushed += 1
        if t in keep:
            m = max(1, len(np.unique(raws[t])))
            outs[t] = torch.empty((m, row_bytes), dtype=torch.uint8, device="cuda")
            uniqs[t] = torch.empty(m, dtype=ses.torch_id, device="cuda")
            seqs.append(ses.gather(None if window else dev[t], outs[t], uniqs[t]))
        else:
            seqs.append(ses.gather(None if window else dev[t], scratch[t & 1], uq_scratch))
        if t >= 40:
            stats[t - 40] = ses.stats(seqs[t - 40])
    torch.cuda.synchronize()
    for t in range(max(0, len(raws) - 40), len(raws)):
        stats[t] = ses.stats(seqs[t])
    return outs, uniqs, stats


def drive_merged(ses, torch, raws, window, row_bytes, k=32, keep=None, cap_rows=None):
    """The same protocol through gids_gather_many, k steps per call (each pushes the list that keeps the window
    full and gathers the head), as bench.py --many issues them; the minibatches in `keep` (all of them when None)
    keep their tensors, the others write to a ring of 2 k buffers of cap_rows rows."""
    dev = [ses.to_device(r) for r in raws]
    n_b = len(raws)
    keep = set(range(n_b)) if keep is None else keep
    ring = [] if len(keep) == n_b else [(torch.empty((cap_rows, row_bytes), dtype=torch.uint8, device="cuda"),
                                         torch.empty(cap_rows, dtype=ses.torch_id, device="cuda")) for _ in range(2 * k)]
    outs = {t: torch.empty((max(1, len(np.unique(raws[t]))), row_bytes), dtype=torch.uint8, device="cuda") for t in keep}
    uniqs = {t: torch.empty(outs[t].shape[0], dtype=ses.torch_id, device="cuda") for t in keep}
    for t in range(n_b):
        if t not in keep:
            outs[t], uniqs[t] = ring[t % (2 * k)]
    stats, pushed, calls = {}, 0, []
    push_stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    while pushed < min(n_b, window):                          # the look-ahead, before the first merged call
        ses.push(dev[pushed], stream=push_stream)
        pushed += 1
    t = 0
    while t < n_b:
        kk = min(k, n_b - t)
        pushes = []
        for i in range(kk):
            if pushed < n_b and pushed <= t + i + window:
                pushes.append(dev[pushed])
                pushed += 1
            else:
                pushes.append(None)
        seq0 = ses.gather_many(pushes, [outs[t + i] for i in range(kk)], [uniqs[t + i] for i in range(kk)],
                               push_stream=push_stream)
        if calls:                                             # the counters of the call before, while this one runs
            t0, k0, s0 = calls[-1]                            # (the library keeps those of the last 64 gathers)
            for i in range(k0):
                stats[t0 + i] = ses.stats(s0 + i)
        calls.append((t, kk, seq0))
        t += kk
    torch.cuda.synchronize()
    t0, k0, s0 = calls[-1]
    for i in range(k0):
        stats[t0 + i] = ses.stats(s0 + i)
    return outs, uniqs, stats


def rows_equal_store(out_dev, u, store_np, chunk=1 << 17):
    """Every gathered row against its row of the host table, the plain definition of the gather."""
    for lo in range(0, len(u), chunk):
        hi = min(len(u), lo + chunk)
        got = out_dev[lo:hi].cpu().numpy()
        if not np.array_equal(got, store_np[u[lo:hi]]):
            bad = np.flatnonzero((got != store_np[u[lo:hi]]).any(axis=1))
            return f"{len(bad)} rows differ, first at j={lo + int(bad[0])} (ID {int(u[lo + bad[0]])})"
    return ""


def store_equals_closed_form(oracle_mod, cfg, store_np, table, n_sample=1500):
    """Pins the table that the definition above refers to: sampled rows (first, last, random) against the
    oracle's own feature formula."""
    rng = np.random.default_rng(cfg.seed & 0xFFFF)
    ids = np.unique(np.concatenate([[0, 1, cfg.n_nodes - 1], rng.integers(0, cfg.n_nodes, n_sample)]))
    want = oracle_mod.feat_rows(cfg.seed, ids, cfg.dim, table).view(np.uint8).reshape(len(ids), -1)
    assert np.array_equal(store_np[ids], want), "the host table differs from the closed-form feature rows"


@pytest.mark.parametrize("merged", [False, True])
def test_medium_full_size(oracle_mod, merged):
    """merged: the same 200 minibatches through gids_gather_many, 32 steps per call (the merged kernels, the
    classification on the library's internal stream)."""
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
    keep = set(range(n_b))                                    # the whole tensor of every minibatch
    with GatherSession(cfg.n_nodes, cfg.row_bytes, np.int64, cfg.cache_lines, cfg.ways, cfg.line_bytes,
                       cfg.window, 1 if merged else 0) as ses:
        wl.fill_store(cfg.seed, cfg.n_nodes, cfg.dim, table, ses.store_address())
        store_equals_closed_form(oracle_mod, cfg, ses.store_view(), table)
        ses.pin_hot(hot)
        if merged:
            outs, uniqs, stats_of = drive_merged(ses, torch, raws, cfg.window, cfg.row_bytes)
        else:
            outs, uniqs, stats_of = drive(ses, torch, raws, cfg.window, cap, cfg.row_bytes, keep)
        sim = oracle_mod.Sim(cfg.n_nodes, cfg.cache_lines, cfg.ways, cfg.window, cfg.row_bytes, cfg.line_bytes,
                             ses.store_view())
        sim.set_hot(hot)
        pushed = 0
        for t, raw in enumerate(raws):
            while pushed < n_b and pushed <= t + cfg.window:
                sim.push(raws[pushed])
                pushed += 1
            u, rows, stats = sim.gather(raw)
            st = stats_of[t]
            assert st.as_tuple() == tuple(int(x) for x in stats), (t, st.as_tuple(), stats.tolist())
            assert np.array_equal(uniqs[t][:len(u)].cpu().numpy(), u)
            assert np.array_equal(outs[t][:len(u)].cpu().numpy(), rows), f"minibatch {t}"
            if t % 50 == 49:
                print(f"[fullsize medium] {t + 1} minibatches: counters, ID lists and whole tensors equal", flush=True)
        tags, stamps = ses.snapshot()
        assert np.array_equal(tags, sim.tags) and np.array_equal(stamps, sim.stamps)
        if merged:
            import paper_2306_16384_amd as gids
            assert gids.gids_cache_many_calls(ses.cache)[1] == 0


def pinnable(cfg_name, sizes):
    """The configuration at the first of `sizes` whose store this box can pin; returns (cfg, store handle)."""
    import paper_2306_16384_amd as gids
    for n_nodes in sizes:
        cfg = CONFIGS[cfg_name] if n_nodes == CONFIGS[cfg_name].n_nodes else wl.scaled(CONFIGS[cfg_name], n_nodes)
        try:
            store = gids.gids_store_create(cfg.n_nodes, cfg.row_bytes, 8)
        except gids.GidsError as e:
            if e.code != gids.GIDS_E_NOMEM:
                raise
            print(f"[fullsize {cfg_name}] cannot pin {cfg.n_nodes * cfg.row_bytes / 1e9:.1f} GB, trying smaller", flush=True)
            continue
        return cfg, store
    pytest.fail(f"cannot pin even {sizes[-1]} rows of host memory")


def sample_lists(g, cfg, n_b, rank_table=None):
    raws = []
    for b in range(n_b):
        raws.append(wl.sample_minibatch(g, cfg.seed, b, cfg.fanouts, cfg.n_seeds, rank_table))
        if b % 100 == 99:
            print(f"[fullsize {cfg.name}] sampled {b + 1} of {n_b} lists", flush=True)
    return raws


def run_big(oracle_mod, cfg, store, store_np, raws, keep, hot=None, after_each=None, window=None, label=None,
            merged_k=0, dedup=False):
    """Counters of every minibatch against the oracle's simulator; on the kept minibatches the distinct-ID list
    and every gathered row; final tags and stamps.  Returns the per-minibatch counters.  merged_k: through
    gids_gather_many, that many steps per call."""
    import torch
    from paper_2306_16384_amd.session import GatherSession
    n_b = len(raws)
    window = cfg.window if window is None else window
    label = label or cfg.name
    cap = max(len(r) for r in raws)                           # raw length bounds the distinct count
    t0 = time.time()
    with GatherSession(cfg.n_nodes, cfg.row_bytes, np.int64, cfg.cache_lines, cfg.ways, cfg.line_bytes,
                       window, 1 if merged_k else 0, store_handle=store) as ses:
        if hot is not None:
            ses.pin_hot(hot)
        if dedup:
            ses.set_group_dedup(True)                         # one transfer per CPU-buffer row and merged call
        if merged_k:
            outs, uniqs, stats_of = drive_merged(ses, torch, raws, window, cfg.row_bytes, merged_k, keep, cap)
        else:
            outs, uniqs, stats_of = drive(ses, torch, raws, window, cap, cfg.row_bytes, keep)
        t_gpu = time.time() - t0
        sim = oracle_mod.Sim(cfg.n_nodes, cfg.cache_lines, cfg.ways, window)      # counts only
        if hot is not None:
            sim.set_hot(hot)
        pushed, n_rows_checked = 0, 0
        for t, raw in enumerate(raws):
            while window and pushed < n_b and pushed <= t + window:
                sim.push(raws[pushed])
                pushed += 1
            u, _, stats = sim.gather(raw, want_rows=False)
            if t % 50 == 49:
                print(f"[fullsize {label}] oracle at minibatch {t + 1} of {n_b}", flush=True)
            st = stats_of[t]
            assert st.as_tuple() == tuple(int(x) for x in stats), (label, t, st.as_tuple(), stats.tolist())
            if after_each:
                after_each(t, st)
            if t in keep:
                assert np.array_equal(uniqs[t][:len(u)].cpu().numpy(), u), (label, t)
                diff = rows_equal_store(outs[t], u, store_np)
                assert not diff, f"{label} minibatch {t}: {diff}"
                n_rows_checked += len(u)
                del outs[t], uniqs[t]
        tags, stamps = ses.snapshot()
        assert np.array_equal(tags, sim.tags) and np.array_equal(stamps, sim.stamps)
        if merged_k:
            import paper_2306_16384_amd as gids
            through = gids.gids_cache_many_calls(ses.cache)
            print(f"[fullsize {label}] merged calls through the merged kernels: {through[0]}, the per-step kernels: {through[1]}", flush=True)
            assert through[0] > through[1], through           # (the first call knows no distinct-per-raw ratio yet)
    print(f"[fullsize {label}] {n_b} minibatches: counters equal; {len(keep)} whole tensors ({n_rows_checked} rows) "
          f"equal the store; tags and stamps equal ({t_gpu:.1f} s GPU leg, {time.time() - t0:.1f} s in all)", flush=True)
    return stats_of


def test_cache_resident_full_size(oracle_mod):
    """The cache-resident configuration at its full size (10 M rows of 3 KiB in 4 KiB lines, a cache that holds
    the whole table): lists that touch every row once, then sampled minibatches, which must all hit."""
    import ctypes as C
    import paper_2306_16384_amd as gids
    cfg, store = pinnable("resident", (10_000_000,))
    try:
        n_b = 200 if EVERY else 40                                # (the configuration names 1000: 19 GB of ID lists)
        print(f"[fullsize resident] N={cfg.n_nodes} lines={cfg.cache_lines} ways={cfg.ways} batches=10+{n_b}", flush=True)
        g = wl.make_graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max, native=True)
        table = wl.normal_table(np.float32)
        ptr = gids.gids_store_host_ptr(store)
        wl.fill_store(cfg.seed, cfg.n_nodes, cfg.dim, table, ptr)
        store_np = np.ctypeslib.as_array((C.c_uint8 * (cfg.n_nodes * cfg.row_bytes)).from_address(ptr)).reshape(cfg.n_nodes, -1)
        store_equals_closed_form(oracle_mod, cfg, store_np, table)
        step = 1_000_000
        raws = [np.arange(b, min(cfg.n_nodes, b + step), dtype=np.int64) for b in range(0, cfg.n_nodes, step)]
        n_pre = len(raws)
        raws += sample_lists(g, cfg, n_b)

        def all_hits_after_coverage(t, st):
            if t >= n_pre:
                assert st.n_miss == 0 and st.n_hit == st.n_unique, (t, st.as_tuple())
            else:
                assert st.n_miss == st.n_unique and st.n_bypass == 0, (t, st.as_tuple())

        # whole tensors: two of the covering lists (fills), then the sampled minibatches (hits) by the usual rule
        keep = {0, n_pre - 1} | kept_minibatches(n_pre + n_b, cfg.window, first=n_pre)
        run_big(oracle_mod, cfg, store, store_np, raws, keep, after_each=all_hits_after_coverage)
    finally:
        gids.gids_store_destroy(store)


# (the tests below share one pinned table; the one above must have released its own before: the box pins 64 GiB)
@pytest.fixture(scope="module")
def big_world(oracle_mod):
    """Large and the skew sweep share one graph, one hot set and one 57 GB table (the configurations differ in
    fanout, seeds, cache shape and window only), pinned and filled once."""
    import torch
    import paper_2306_16384_amd as gids
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (no CPU fallback exists)")
    cfg, store = pinnable("large", (28_000_000, 14_000_000, 7_000_000))
    try:
        print(f"[fullsize] table of {cfg.n_nodes} rows pinned", flush=True)
        g = wl.make_graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max, native=True)
        hot = wl.hot_nodes(g, cfg.cpu_rows)
        table = wl.normal_table(np.float16)
        ptr = gids.gids_store_host_ptr(store)
        wl.fill_store(cfg.seed, cfg.n_nodes, cfg.dim, table, ptr)
        import ctypes as C
        store_np = np.ctypeslib.as_array((C.c_uint8 * (cfg.n_nodes * cfg.row_bytes)).from_address(ptr)).reshape(cfg.n_nodes, -1)
        store_equals_closed_form(oracle_mod, cfg, store_np, table)
        yield dict(cfg=cfg, store=store, store_np=store_np, g=g, hot=hot, lists={})
    finally:
        gids.gids_store_destroy(store)


def test_large_at_benchmark_size(oracle_mod, big_world):
    # the benchmark's node count; a box that pins less host memory runs the same test at half the size
    cfg = big_world["cfg"]
    n_b = CONFIGS["large"].n_batches                          # all 500
    print(f"[fullsize large] N={cfg.n_nodes} lines={cfg.cache_lines} cpu_rows={cfg.cpu_rows} batches={n_b}", flush=True)
    raws = sample_lists(big_world["g"], cfg, n_b)
    run_big(oracle_mod, cfg, big_world["store"], big_world["store_np"], raws, kept_minibatches(n_b, cfg.window),
            hot=big_world["hot"])


@pytest.mark.parametrize("k,dedup", [(8, False), (32, True)])
def test_large_in_merged_calls(oracle_mod, big_world, k, dedup):
    """120 minibatches of Large through gids_gather_many, 8 or 32 steps per call (32: classified 16 steps per
    launch): the pushed lists go through the bitmap in device memory, the classification keeps its lists in LDS
    and the sets' state in memory.  dedup: a CPU-buffer row that several steps of a call need crosses the link
    once."""
    cfg = big_world["cfg"]
    n_b = 120
    if "large120" not in big_world["lists"]:
        big_world["lists"]["large120"] = sample_lists(big_world["g"], cfg, n_b)
    raws = big_world["lists"]["large120"]
    run_big(oracle_mod, cfg, big_world["store"], big_world["store_np"], raws, kept_minibatches(n_b, cfg.window),
            hot=big_world["hot"], merged_k=k, dedup=dedup, label=f"large merged/{k}{'/dedup' if dedup else ''}")


@pytest.mark.parametrize("dedup", [False, True])
def test_skew_in_merged_calls(oracle_mod, big_world, dedup):
    """160 minibatches of the skew configuration (Zipf 0.8 seeds, depth 4) through gids_gather_many, 32 steps per
    call; dedup: a CPU-buffer row that several steps of a call need crosses the link once."""
    base = big_world["cfg"]
    cfg = wl.scaled(CONFIGS["skew"], base.n_nodes)
    n_b = 160
    if "skew160" not in big_world["lists"]:
        rank_table = wl.synth.zipf_rank_table(cfg.n_nodes, 0.8)
        big_world["lists"] = {"skew160": sample_lists(big_world["g"], cfg, n_b, rank_table)}
    raws = big_world["lists"]["skew160"]
    run_big(oracle_mod, cfg, big_world["store"], big_world["store_np"], raws, kept_minibatches(n_b, cfg.window),
            hot=big_world["hot"], merged_k=32, dedup=dedup, label=f"skew merged{'/dedup' if dedup else ''}")


SKEW_S = (0.0, 0.8, 1.2)
SKEW_W = (0, 4, 16)
RESULTS = os.environ.get("GIDS_RESULTS_DIR")               # where the measured points are appended, if anywhere


def skew_point(oracle_mod, big_world, s_exp, window, cache_lines, n_b, tag):
    base = big_world["cfg"]
    cfg = wl.scaled(CONFIGS["skew"], base.n_nodes)
    if cache_lines:
        from dataclasses import replace
        cfg = replace(cfg, cache_lines=cache_lines)
    key = (s_exp, n_b)
    if key not in big_world["lists"]:                         # one list sequence per Zipf exponent, shared by its depths
        rank_table = wl.synth.zipf_rank_table(cfg.n_nodes, s_exp)
        big_world["lists"] = {key: sample_lists(big_world["g"], cfg, n_b, rank_table)}
    raws = big_world["lists"][key]
    label = f"skew/{tag}/s{s_exp}/W{window}"
    print(f"[fullsize {label}] N={cfg.n_nodes} lines={cfg.cache_lines} ways={cfg.ways} batches={n_b}", flush=True)
    stats = run_big(oracle_mod, cfg, big_world["store"], big_world["store_np"], raws,
                    kept_minibatches(n_b, window) if not cache_lines else {0, n_b // 2, n_b - 1},
                    hot=big_world["hot"], window=window, label=label)
    tail = [stats[t] for t in range(n_b // 2, n_b)]           # second half: past the cold start
    uniq = sum(s.n_unique for s in tail)
    cold = sum(s.n_unique - s.n_cpu_hit for s in tail)        # what reaches the GPU cache
    point = {"zipf_s": s_exp, "window": window, "cache_lines": cfg.cache_lines, "minibatches": n_b,
             "hit_rate": sum(s.n_hit for s in tail) / uniq, "cpu_buffer_rate": sum(s.n_cpu_hit for s in tail) / uniq,
             "hit_rate_of_cache_traffic": sum(s.n_hit for s in tail) / max(1, cold),
             "bypass_rate": sum(s.n_bypass for s in tail) / uniq}
    print(f"[fullsize {label}] {json.dumps(point)}", flush=True)
    if RESULTS:
        try:
            os.makedirs(RESULTS, exist_ok=True)
            with open(os.path.join(RESULTS, "skew_parity_points.jsonl"), "a") as f:
                f.write(json.dumps(dict(point, tag=tag)) + "\n")
        except OSError:
            pass
    return point


@pytest.mark.parametrize("s_exp", SKEW_S)
def test_skew_sweep_at_benchmark_size(oracle_mod, big_world, s_exp):
    """The nine points of the skew sweep (seed Zipf s x window depth; 16 ways) at the node count the benchmark
    runs, each a cache of its own over the shared table."""
    n_b = CONFIGS["skew"].n_batches                           # all 300
    for window in SKEW_W:
        skew_point(oracle_mod, big_world, s_exp, window, 0, n_b, "config")


@pytest.mark.parametrize("s_exp", SKEW_S)
def test_skew_sweep_under_eviction_pressure(oracle_mod, big_world, s_exp):
    """The same nine points with a cache of a few minibatches' misses (2,048 sets x 16 ways), so that lines are
    evicted inside the run and the window has something to protect (whether hits rise with the depth is the
    workload's business, Section 4.5; parity is what is asserted).  The points are recorded for the report."""
    n_b = 96
    pts = [skew_point(oracle_mod, big_world, s_exp, window, 2048 * 16, n_b, "pressure") for window in SKEW_W]
    assert all(p["hit_rate"] > 0 for p in pts)
