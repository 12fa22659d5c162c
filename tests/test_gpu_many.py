"""gids_gather_many: k steps of the steady-state loop (push one list, gather the
window's head) in one call, as one accumulator group.  Outputs, counters and
cache state must be those of the oracle fed the same steps one by one."""
import os

import numpy as np
import pytest

import workload as wl
from workload import CONFIGS

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (no CPU fallback exists)")
    import paper_2306_16384_amd as gids
    from paper_2306_16384_amd.session import GatherSession
    gids.lib()
    return torch, gids, GatherSession


def with_env(knobs, make):
    """knobs: name -> value, None = not set"""
    old = {k: os.environ.get(k) for k in knobs}
    for k, v in knobs.items():
        if v is None:
            os.environ.pop(k, None)
        else:
            os.environ[k] = v
    try:
        return make()
    finally:
        for k, v in old.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v


def run_many(gpu, oracle, feats, batches, *, id_dtype, lines, ways, window, ks, hot=None, policy=None, pipeline="0",
             fuse=None, pool=None, resident=None, meta_min=None, list_max=None, dedup=False, chunk=None, exact_again=False, expect_merged=None, label=""):
    """ks: the sizes of the merged calls, in order (0 = one plain push + gather step in between);
    cycles until every list is gathered."""
    torch, gids, GatherSession = gpu
    n_rows = feats.shape[0]
    feats_u8 = np.ascontiguousarray(feats).view(np.uint8).reshape(n_rows, -1)
    R = feats_u8.shape[1]
    n_b = len(batches)
    print(f"[many {label}] rows={n_rows} R={R} lines={lines} ways={ways} W={window} pipe={pipeline} fuse={fuse} "
          f"pool={pool} resident={resident} ks={ks}", flush=True)
    sim = oracle.Sim(n_rows, lines, ways, window, R, R, feats_u8)
    if hot is not None:
        sim.set_hot(hot)
    if policy is not None:
        sim.set_policy(*policy)
    want, pushed = [], 0
    for t, raw in enumerate(batches):
        while window and pushed < n_b and pushed <= t + window:
            sim.push(batches[pushed])
            pushed += 1
        want.append(sim.gather(raw))
    knobs = {"GIDS_PIPELINE": pipeline if pipeline in ("0", "1") else None}
    if fuse is not None:
        knobs["GIDS_FUSE"] = fuse
    if pool is not None:
        knobs["GIDS_MANY_POOL"] = pool
    if resident is not None:
        knobs["GIDS_MANY_RESIDENT"] = resident
    knobs["GIDS_MANY_PIPELINE_MIN"] = meta_min
    knobs["GIDS_MANY_LIST_MAX"] = list_max
    knobs["GIDS_MANY_CHUNK"] = chunk
    ses = with_env(knobs, lambda: GatherSession(n_rows, R, id_dtype, lines, ways, R, window, 1000))
    with ses:
        ses.store_view()[:] = feats_u8
        if hot is not None:
            ses.pin_hot(hot)
        if policy is not None:
            ses.set_policy(*policy)
        if dedup:
            ses.set_group_dedup(True)
        dev = [ses.to_device(b) for b in batches]
        torch.cuda.synchronize()
        push_stream = torch.cuda.Stream() if pipeline in ("1", None) else None
        outs = [torch.full((max(len(b), 1), R), 0xA5, dtype=torch.uint8, device="cuda") for b in batches]
        uqs = [torch.full((max(len(b), 1),), -7, dtype=ses.torch_id, device="cuda") for b in batches]
        seq_of, expect_acc, again_of = {}, {}, {}
        pushed = 0
        if window == 0:
            pass                                              # depth 0: every step pushes its own list just before
        else:
            while pushed < min(n_b, window):                  # the look-ahead, filled by plain pushes
                ses.push(dev[pushed], stream=push_stream)
                pushed += 1
        t, call = 0, 0
        while t < n_b:
            k = ks[call % len(ks)]
            call += 1
            if k == 0:                                        # a plain step between merged calls
                if pushed < n_b and pushed <= t + window:
                    ses.push(dev[pushed], stream=push_stream)
                    pushed += 1
                seq_of[t] = ses.gather(None, outs[t], uqs[t])
                expect_acc[t] = None
                t += 1
                continue
            k = min(k, n_b - t)
            pushes = []
            for i in range(k):
                if pushed < n_b and pushed <= t + i + window:
                    pushes.append(dev[pushed])
                    pushed += 1
                else:
                    pushes.append(None)
            seq0 = ses.gather_many(pushes, outs[t:t + k], uqs[t:t + k], push_stream=push_stream)
            rows = 0
            seen_hot = set()                                  # CPU-buffer rows the call's earlier steps already fetch
            for i in range(k):
                if dedup and hot is not None:
                    mine = set(np.intersect1d(want[t + i][0], hot).tolist())
                    again_of[t + i] = len(mine & seen_hot)
                    seen_hot |= mine
                else:
                    again_of[t + i] = 0
                seq_of[t + i] = seq0 + i
                rows += len(want[t + i][0])
                expect_acc[t + i] = (0, 1) if i == k - 1 else (rows, 0)
            t += k
        ses.flush()
        torch.cuda.synchronize()
        for t in range(n_b):
            u, rows, stats = want[t]
            st = ses.stats(seq_of[t])
            assert st.status == 0
            assert st.as_tuple() == tuple(int(x) for x in stats), (label, t, st.as_tuple(), stats.tolist())
            if expect_acc[t] is not None:
                assert (st.n_pending, st.flushed) == expect_acc[t], (label, t, st.n_pending, st.flushed, expect_acc[t])
            # (plain steps between the calls belong to groups of their own: not modelled here; a workgroup that
            # had to read the lists from memory fetches every row: equality only where none did)
            if t in again_of and exact_again:
                assert st.n_cpu_again == again_of[t], (label, t, st.n_cpu_again, again_of[t])
            elif t in again_of:
                assert st.n_cpu_again <= again_of[t], (label, t, st.n_cpu_again, again_of[t])
            elif not dedup:
                assert st.n_cpu_again == 0
            m = len(u)
            assert np.array_equal(uqs[t][:m].cpu().numpy(), u.astype(ses.id_dtype)), (label, t)
            assert np.array_equal(outs[t][:m].cpu().numpy(), rows), f"{label} minibatch {t}: gathered rows differ"
            if m < outs[t].shape[0]:
                assert bool((outs[t][m:] == 0xA5).all())
        tags, stamps = ses.snapshot()
        assert np.array_equal(tags, sim.tags), label
        assert np.array_equal(stamps, sim.stamps), label
        merged, per_step = gids.gids_cache_many_calls(ses.cache)
        print(f"[many {label}] calls through the merged kernels: {merged}, through the per-step kernels: {per_step}", flush=True)
        if expect_merged is True:
            assert merged > 0 and per_step == 0, (label, merged, per_step)
        if expect_merged is False:
            assert merged == 0 and per_step > 0, (label, merged, per_step)
        return merged, per_step


def zipf_lists(rng, n, n_b, size, a=1.2):
    return [np.minimum(rng.zipf(a, size=int(rng.integers(size // 2, size + 1))) - 1, n - 1).astype(np.int64)
            for _ in range(n_b)]


@pytest.mark.parametrize("pipeline", ["0", "1"])
def test_tiny_config_in_merged_calls(gpu, oracle_mod, pipeline):
    cfg = CONFIGS["tiny"]
    g = wl.make_graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max)
    table = wl.normal_table(np.float32)
    feats = wl.feature_rows(cfg.seed, np.arange(cfg.n_nodes), cfg.dim, table)
    hot = wl.hot_nodes(g, cfg.cpu_rows)
    batches = [wl.sample_minibatch(g, cfg.seed, b, cfg.fanouts, cfg.n_seeds) for b in range(48)]
    for ks in ([8], [1, 3, 0, 32, 2], [32]):
        run_many(gpu, oracle_mod, feats, batches, id_dtype=np.int32, lines=cfg.cache_lines, ways=cfg.ways,
                 window=cfg.window, ks=ks, hot=hot, pipeline=pipeline, expect_merged=True, label=f"tiny/{ks}")


@pytest.mark.parametrize("ways,window,id_dtype,policy", [(1, 0, np.int64, None), (2, 1, np.int32, None), (4, 3, np.int64, (1, 7)),
                                                         (8, 9, np.int32, None), (16, 2, np.int64, (1, 3)), (64, 2, np.int64, None)])
def test_merged_calls_over_shapes(gpu, oracle_mod, ways, window, id_dtype, policy):
    """Associativity (64 ways takes the per-step kernels), window depths beyond and below the call size, both ID
    widths and both policies; a small cache, so that lines are hit, evicted and refilled inside one call."""
    rng = np.random.default_rng(500 + ways + window)
    n = 3000
    feats = rng.integers(0, 256, size=(n, 128), dtype=np.uint8)
    batches = zipf_lists(rng, n, 40, 500)
    batches[7] = np.array([5], dtype=np.int64)
    batches[11] = np.arange(n, dtype=np.int64)                 # the whole table
    for pipeline in ("0", "1"):
        run_many(gpu, oracle_mod, feats, batches, id_dtype=id_dtype, lines=ways * 11, ways=ways, window=window,
                 ks=[5, 0, 13, 1], hot=rng.choice(n, 40, replace=False), policy=policy, pipeline=pipeline,
                 expect_merged=ways <= 16, label=f"ways{ways}/W{window}")


@pytest.mark.parametrize("pool,resident", [("0", None), ("3000", None), ("14000", None), ("14000", "0"), (None, "0")])
def test_merged_calls_with_little_or_no_lds(gpu, oracle_mod, pool, resident):
    """A classifying workgroup keeps its own entries of every list in LDS, and the state of its sets as well when
    that fits; one whose share of some list does not fit reads the lists from memory in every phase instead.  No
    LDS: all of them do; 14,000 bytes: about as many places as the expected share, so workgroups of both kinds run
    side by side in one launch; resident 0: the lists in LDS, the sets' state in device memory."""
    cfg = CONFIGS["tiny"]
    g = wl.make_graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max)
    table = wl.normal_table(np.float32)
    feats = wl.feature_rows(cfg.seed, np.arange(cfg.n_nodes), cfg.dim, table)
    hot = wl.hot_nodes(g, cfg.cpu_rows)
    batches = [wl.sample_minibatch(g, cfg.seed, b, cfg.fanouts, cfg.n_seeds) for b in range(40)]
    run_many(gpu, oracle_mod, feats, batches, id_dtype=np.int32, lines=cfg.cache_lines, ways=cfg.ways,
             window=cfg.window, ks=[32, 3, 0, 5], hot=hot, pool=pool, resident=resident, expect_merged=True,
             label="tiny")
    rng = np.random.default_rng(91)
    n = 3000
    feats = rng.integers(0, 256, size=(n, 128), dtype=np.uint8)
    batches = zipf_lists(rng, n, 30, 500)
    batches[9] = np.arange(n, dtype=np.int64)
    for policy in (None, (1, 5)):
        run_many(gpu, oracle_mod, feats, batches, id_dtype=np.int64, lines=8 * 11, ways=8, window=3, ks=[7, 0, 12],
                 hot=rng.choice(n, 40, replace=False), pool=pool, resident=resident, policy=policy, pipeline="1",
                 expect_merged=True, label="small cache")


@pytest.mark.parametrize("meta_min", [None, "16"])
@pytest.mark.parametrize("own_push_stream", [True, False])
def test_long_and_short_merged_calls_and_plain_steps_take_turns(gpu, oracle_mod, own_push_stream, meta_min):
    """On a small cache merged calls classify on the library's internal stream (by default from two steps on, here
    also from 16 on), shorter ones and plain gathers on the caller's.  Every change of stream between consecutive
    calls is in here."""
    cfg = CONFIGS["tiny"]
    g = wl.make_graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max)
    table = wl.normal_table(np.float32)
    feats = wl.feature_rows(cfg.seed, np.arange(cfg.n_nodes), cfg.dim, table)
    hot = wl.hot_nodes(g, cfg.cpu_rows)
    batches = [wl.sample_minibatch(g, cfg.seed, b, cfg.fanouts, cfg.n_seeds) for b in range(60)]
    run_many(gpu, oracle_mod, feats, batches, id_dtype=np.int32, lines=cfg.cache_lines, ways=cfg.ways,
             window=cfg.window, ks=[16, 3, 0, 20, 0, 17, 2], hot=hot,
             pipeline=None if own_push_stream else "unset-one-stream", meta_min=meta_min, expect_merged=True,
             label="default streams")


@pytest.mark.parametrize("own_push_stream", [True, False])
def test_two_thousand_minibatches_in_merged_calls(gpu, oracle_mod, own_push_stream):
    """A long run of merged calls on a small cache: the rings of events and counters wrap many times, every window
    slot and both sets of group lists are reused hundreds of times, calls of 32, 7 and 19 steps take turns; the
    counters of every minibatch (read one call behind), sampled tensors and the final tags and stamps must equal
    the oracle's."""
    torch, gids, GatherSession = gpu
    cfg = CONFIGS["tiny"]
    g = wl.make_graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max)
    table = wl.normal_table(np.float32)
    feats = wl.feature_rows(cfg.seed, np.arange(cfg.n_nodes), cfg.dim, table).view(np.uint8).reshape(cfg.n_nodes, -1)
    hot = wl.hot_nodes(g, cfg.cpu_rows)
    base = [wl.sample_minibatch(g, cfg.seed, b, cfg.fanouts, cfg.n_seeds) for b in range(41)]
    n_b, W = 2000, 6
    lists = [base[(9 * t) % 41] for t in range(n_b)]
    sim = oracle_mod.Sim(cfg.n_nodes, cfg.cache_lines, cfg.ways, W, cfg.row_bytes, cfg.line_bytes, feats)
    sim.set_hot(hot)
    want, pushed = [], 0
    check_rows = set(range(0, n_b, 131)) | {n_b - 1}
    for t in range(n_b):
        while pushed < n_b and pushed <= t + W:
            sim.push(lists[pushed])
            pushed += 1
        want.append(sim.gather(lists[t], want_rows=t in check_rows))
    with GatherSession(cfg.n_nodes, cfg.row_bytes, np.int32, cfg.cache_lines, cfg.ways, cfg.line_bytes, W, 1) as ses:
        ses.store_view()[:] = feats
        ses.pin_hot(hot)
        dev = [ses.to_device(b) for b in base]
        cap = max(len(b) for b in base)
        ps = torch.cuda.Stream() if own_push_stream else None
        # an output must stay untouched until its call has moved its rows: two calls' worth of buffers
        ring = [torch.empty((cap, cfg.row_bytes), dtype=torch.uint8, device="cuda") for _ in range(64)]
        uqs = [torch.empty(cap, dtype=torch.int32, device="cuda") for _ in range(64)]
        kept, pushed = {}, 0
        while pushed < W:
            ses.push(dev[(9 * pushed) % 41], stream=ps)
            pushed += 1
        t, call, before = 0, 0, None
        while t < n_b:
            k = min((32, 7, 19)[call % 3], n_b - t)
            call += 1
            pushes, outs, uq = [], [], []
            for i in range(k):
                if pushed < n_b and pushed <= t + i + W:
                    pushes.append(dev[(9 * pushed) % 41])
                    pushed += 1
                else:
                    pushes.append(None)
                if t + i in check_rows:
                    kept[t + i] = (torch.empty((cap, cfg.row_bytes), dtype=torch.uint8, device="cuda"),
                                   torch.empty(cap, dtype=torch.int32, device="cuda"))
                    outs.append(kept[t + i][0])
                    uq.append(kept[t + i][1])
                else:
                    outs.append(ring[(t + i) % 64])
                    uq.append(uqs[(t + i) % 64])
            seq0 = ses.gather_many(pushes, outs, uq, push_stream=ps)
            if before is not None:                            # the counters of the call before, while this one runs
                t0, k0, s0 = before
                for i in range(k0):
                    assert ses.stats(s0 + i).as_tuple() == tuple(int(x) for x in want[t0 + i][2]), t0 + i
            before = (t, k, seq0)
            t += k
        t0, k0, s0 = before
        for i in range(k0):
            assert ses.stats(s0 + i).as_tuple() == tuple(int(x) for x in want[t0 + i][2]), t0 + i
        torch.cuda.synchronize()
        for t in sorted(check_rows):
            u, rows, _ = want[t]
            assert np.array_equal(kept[t][1][:len(u)].cpu().numpy(), u.astype(np.int32)), t
            assert np.array_equal(kept[t][0][:len(u)].cpu().numpy(), rows), t
        tags, stamps = ses.snapshot()
        assert np.array_equal(tags, sim.tags) and np.array_equal(stamps, sim.stamps)
        assert gids.gids_cache_many_calls(ses.cache)[1] == 0


N_RANDOM = int(os.environ.get("GIDS_MANY_RANDOM_CASES", "32"))
RANDOM_TALLY = [0, 0]                                         # calls through the merged kernels / the per-step kernels


@pytest.mark.parametrize("case", range(N_RANDOM))
def test_random_merged_calls(gpu, oracle_mod, case):
    """Seeded random geometry, window, list shapes, call sizes and the library's knobs for the merged kernels (the
    draw is printed, so a failure names its case)."""
    rng = np.random.default_rng(31_000 + case)
    n = int(rng.choice([64, 65, 1000, 4097, 30_011, 200_003, 2_000_003]))
    ways = int(rng.choice([1, 2, 4, 8, 16]))
    n_sets = int(rng.integers(1, max(2, n // (ways * int(rng.integers(1, 60))) + 2)))
    row_bytes = int(rng.choice([16, 64, 512, 1040]))
    window = int(rng.choice([0, 1, 2, 4, 9, 20]))
    id_dtype = np.int32 if rng.random() < 0.5 else np.int64
    n_hot = int(rng.integers(0, max(1, n // 8)))
    size = int(rng.integers(1, min(3 * n, 20_000)))
    a = float(rng.choice([1.05, 1.3, 2.0]))
    n_b = int(rng.integers(4, 60))
    batches = []
    for _ in range(n_b):
        m = int(rng.integers(0, size + 1))
        kind = rng.random()
        if kind < 0.4:
            b = np.minimum(rng.zipf(a, size=m) - 1, n - 1)
        elif kind < 0.8:
            b = rng.integers(0, n, size=m)
        else:                                                 # a run of neighbouring IDs: every set gets its share
            lo = int(rng.integers(0, n))
            b = (lo + np.arange(m)) % n
        batches.append(b.astype(np.int64))
    ks = [int(k) for k in rng.choice([0, 1, 2, 5, 16, 17, 32], size=int(rng.integers(1, 6)))]
    if all(k == 0 for k in ks):
        ks.append(32)
    pipeline = [None, "0", "1", "unset-one-stream"][case % 4]
    pool, resident = [(None, None), (None, "0"), ("0", None), (str(int(rng.integers(200, 40_000))), None),
                      (None, None)][case % 5]
    feats = rng.integers(0, 256, size=(n, row_bytes), dtype=np.uint8)
    merged, per_step = run_many(gpu, oracle_mod, feats, batches, id_dtype=id_dtype, lines=ways * n_sets, ways=ways,
                                window=window, ks=ks, hot=rng.choice(n, n_hot, replace=False) if n_hot else None,
                                policy=(1, case) if rng.random() < 0.3 else None, pipeline=pipeline, pool=pool,
                                resident=resident, meta_min=[None, "16", "0"][case % 3], dedup=case % 2 == 1,
                                chunk=[None, None, "3", "8"][case % 4] if resident == "0" else None,
                                label=f"random{case}")
    RANDOM_TALLY[0] += merged
    RANDOM_TALLY[1] += per_step


def test_random_merged_calls_took_both_kinds_of_kernels():
    """(runs after the random cases: most of their calls must have gone through the merged kernels)"""
    if sum(RANDOM_TALLY) == 0:
        pytest.skip("the random cases did not run in this process")
    assert RANDOM_TALLY[0] > RANDOM_TALLY[1] > 0, RANDOM_TALLY


@pytest.mark.parametrize("resident", [None, "0"])
def test_cpu_buffer_rows_cross_the_link_once_per_call(gpu, oracle_mod, resident):
    """gids_cache_set_group_dedup: a large CPU buffer and heavily overlapping lists, so that most CPU-buffer rows of
    a call are needed by several of its steps; outputs, counters and cache state must not change.  With the sets'
    state in LDS and in device memory; switching it on and off between calls."""
    torch, gids, GatherSession = gpu
    rng = np.random.default_rng(5150)
    n = 20_000
    feats = rng.integers(0, 256, size=(n, 256), dtype=np.uint8)
    hot = rng.choice(n, 6000, replace=False)
    batches = [np.concatenate([rng.choice(hot, 1500), rng.integers(0, n, size=800)]).astype(np.int64) for _ in range(50)]
    for pipeline in ("0", "1"):
        run_many(gpu, oracle_mod, feats, batches, id_dtype=np.int64, lines=4 * 256, ways=4, window=5, ks=[32, 0, 7, 2],
                 hot=hot, pipeline=pipeline, resident=resident, dedup=True, exact_again=True, expect_merged=True,
                 label="dedup")
    with GatherSession(n, 256, np.int64, 1024, 4, 256, 0, 1) as ses:            # on, off and on again
        ses.store_view()[:] = feats
        ses.pin_hot(hot)
        dev = [ses.to_device(b) for b in batches[:6]]
        outs = [torch.zeros((len(b), 256), dtype=torch.uint8, device="cuda") for b in batches[:6]]
        uqs = [torch.zeros(len(b), dtype=torch.int64, device="cuda") for b in batches[:6]]
        for on, lo in ((True, 0), (False, 2), (True, 4)):
            ses.set_group_dedup(on)
            ses.gather_many(dev[lo:lo + 2], outs[lo:lo + 2], uqs[lo:lo + 2])
        torch.cuda.synchronize()
        for t in range(6):
            u = np.unique(batches[t])
            assert np.array_equal(uqs[t][:len(u)].cpu().numpy(), u)
            assert np.array_equal(outs[t][:len(u)].cpu().numpy(), feats[u])
    with GatherSession(n, 256, np.int64, 1024, 4, 256, 0) as ses:               # no accumulator
        with pytest.raises(gids.GidsError) as e:
            ses.set_group_dedup(True)
        assert e.value.code == gids.GIDS_E_INVAL


@pytest.mark.parametrize("chunk,dedup", [("4", False), ("5", True), ("16", True)])
def test_a_call_classified_in_several_launches(gpu, oracle_mod, chunk, dedup):
    """Where the sets' state stays in device memory a call whose lists do not fit a workgroup's LDS together is
    classified a few steps per launch, the group staying open in between (here forced: GIDS_MANY_CHUNK).  Lines
    installed in one launch and hit, evicted or installed again in a later one of the same call; n_pending across
    the launches; CPU-buffer rows remembered from launch to launch."""
    rng = np.random.default_rng(626)
    n = 9000
    feats = rng.integers(0, 256, size=(n, 128), dtype=np.uint8)
    hot = rng.choice(n, 2000, replace=False)
    batches = [np.concatenate([rng.choice(hot, 400), np.minimum(rng.zipf(1.3, size=700) - 1, n - 1)]).astype(np.int64)
               for _ in range(56)]
    for pipeline in ("0", "1"):
        run_many(gpu, oracle_mod, feats, batches, id_dtype=np.int64, lines=8 * 16, ways=8, window=3, ks=[32, 0, 13, 7],
                 hot=hot, pipeline=pipeline, resident="0", chunk=chunk, dedup=dedup, exact_again=True,
                 expect_merged=True, label=f"chunks of {chunk}")


def test_merged_calls_through_the_per_step_kernels(gpu, oracle_mod):
    """The same calls with the merged kernels switched off (what a large table gets): one group per call."""
    rng = np.random.default_rng(77)
    n = 5000
    feats = rng.integers(0, 256, size=(n, 64), dtype=np.uint8)
    batches = zipf_lists(rng, n, 30, 700)
    for pipeline in ("0", "1"):
        run_many(gpu, oracle_mod, feats, batches, id_dtype=np.int64, lines=256, ways=4, window=4, ks=[6, 0, 9],
                 hot=rng.choice(n, 60, replace=False), pipeline=pipeline, fuse="0", expect_merged=False, label="per-step")


@pytest.mark.parametrize("n", [600_000, 1_500_000, 5_000_000])
def test_tables_beyond_64_kib_of_bitmap(gpu, oracle_mod, n):
    """600,000 rows: the merged dedup's LDS bitmap needs more than the default 64 KiB of a workgroup; 1,500,000
    and 5,000,000 rows: more than a workgroup can have, the pushed lists of a call are deduplicated through the
    bitmap in device memory, one after the other.  Then a list beyond the merged kernels' length limit (set to
    10,000 here): the calls that read it take the per-step kernels, the others do not."""
    rng = np.random.default_rng(78)
    feats = rng.integers(0, 256, size=(n, 16), dtype=np.uint8)
    batches = [rng.integers(0, n, size=3000) for _ in range(12)]
    batches[5] = rng.integers(0, n, size=20_000)
    batches[8] = np.minimum(rng.zipf(1.2, size=9000) - 1, n - 1)
    for pipeline in ("0", "1"):
        run_many(gpu, oracle_mod, feats, batches, id_dtype=np.int64, lines=1024, ways=8, window=2, ks=[4, 0, 3],
                 pipeline=pipeline, expect_merged=True, label=f"{n} rows")
    merged, per_step = run_many(gpu, oracle_mod, feats, batches, id_dtype=np.int64, lines=1024, ways=8, window=2,
                                ks=[4], list_max="10000", label=f"{n} rows, no lists beyond 10,000")
    assert merged > 0 and per_step > 0


def test_merged_call_errors(gpu):
    torch, gids, GatherSession = gpu
    feats = np.arange(200 * 64, dtype=np.uint8).reshape(200, 64)
    out = [torch.zeros((8, 64), dtype=torch.uint8, device="cuda") for _ in range(3)]
    with GatherSession(200, 64, np.int64, 16, 4, 64, 1) as s:      # no accumulator
        with pytest.raises(gids.GidsError) as e:
            s.gather_many([s.to_device([1])], out[:1])
        assert e.value.code == gids.GIDS_E_INVAL
    with GatherSession(200, 64, np.int64, 16, 4, 64, 1, 100) as s:
        s.store_view()[:] = feats
        with pytest.raises(gids.GidsError) as e:                # nothing buffered and nothing pushed
            s.gather_many([None], out[:1])
        assert e.value.code == gids.GIDS_E_ORDER
        with pytest.raises(gids.GidsError) as e:                # 33 steps
            s.gather_many([None] * 33, [out[0]] * 33)
        assert e.value.code == gids.GIDS_E_INVAL
        assert gids.gids_cache_gathers(s.cache) == 0
        # the second step's output is too small: step 0 stands, steps 1 and 2 report the error
        lists = [s.to_device([1, 2, 3]), s.to_device(np.arange(20)), s.to_device([4])]
        seq0 = s.gather_many(lists, out)
        st0 = s.stats(seq0)
        assert st0.as_tuple() == (3, 0, 0, 3, 0)
        with pytest.raises(gids.GidsError) as e:
            s.stats(seq0 + 1)
        assert e.value.code == gids.GIDS_E_SPACE
        torch.cuda.synchronize()
        assert np.array_equal(out[0][:3].cpu().numpy(), feats[[1, 2, 3]])
    with GatherSession(200, 64, np.int64, 16, 4, 64, 1, 100) as s:     # a pushed ID outside the table
        seq0 = s.gather_many([s.to_device([1, 2]), s.to_device([7, 200])], out[:2])
        with pytest.raises(gids.GidsError) as e:
            s.stats(seq0)
        assert e.value.code == gids.GIDS_E_RANGE
