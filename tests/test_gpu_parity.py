"""Parity of the HIP library (through its C ABI) with the CPU oracle: gathered
tensor, distinct-ID list and per-minibatch hit / CPU-buffer-hit / miss / bypass
counts, all bit-exact, plus the final tag and stamp of every cache line."""
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


def run_case(gpu, oracle, feats, batches, *, id_dtype, lines, ways, line_bytes, window, threshold=0, hot=None,
             use_head=False, with_inverse=False, check_state=True, two_streams=False, policy=None, label="",
             pipeline=None, push_depth0=False, wide_index=False, rows_per_line=1, accum_mode=0, fused=None,
             dedup=False):
    """Feeds the same raw ID lists to both implementations, protocol: keep window + 1 lists buffered.
    pipeline: "0" / "1" forces the library's internal stream off / on for this cache (GIDS_PIPELINE);
    fused: True / False switches the settle kernel (commit + queueing + counters) on / off (GIDS_FUSE);
    push_depth0: at window depth 0, push every list just before its gather."""
    torch, gids, GatherSession = gpu
    n_rows = feats.shape[0]
    feats_u8 = np.ascontiguousarray(feats).view(np.uint8).reshape(n_rows, -1)
    row_bytes = feats_u8.shape[1]
    sim = oracle.Sim(n_rows, lines, ways, window, row_bytes, line_bytes, feats_u8)
    print(f"[case {label}] rows={n_rows} R={row_bytes} L={line_bytes} lines={lines} ways={ways} W={window} "
          f"thr={threshold} ids={np.dtype(id_dtype).name} batches={len(batches)}", flush=True)
    if hot is not None and len(hot):
        sim.set_hot(hot)
    if policy is not None:
        sim.set_policy(*policy)
    if rows_per_line != 1:
        sim.set_rows_per_line(rows_per_line)
    if threshold:
        sim.set_accum(threshold, accum_mode)
    # the oracle's pass, on its own
    want, line_fills, accum, pushed = [], [], [], 0
    for t, raw in enumerate(batches):
        while window and pushed < len(batches) and pushed <= t + window:
            sim.push(batches[pushed])
            pushed += 1
        u, rows, stats, cls = sim.gather(raw, want_cls=True)
        want.append((u, rows, stats))
        accum.append(sim.accum_last)
        line_fills.append(len(np.unique(u[cls == 2] // rows_per_line)))   # distinct store lines among installed misses
    import os
    knobs = {}                                               # environment knobs are read when the cache is created
    if pipeline is not None:
        knobs["GIDS_PIPELINE"] = pipeline
    if wide_index:
        knobs["GIDS_WIDE_INDEX"] = "1"                       # the arithmetic of stores with 2^32 rows and more
    if fused is not None:
        knobs["GIDS_FUSE"] = "1" if fused else "0"          # commit + queueing + counters in one launch, or a kernel each
    old_env = {k: os.environ.get(k) for k in knobs}
    os.environ.update(knobs)
    try:
        ses_cm = GatherSession(n_rows, row_bytes, id_dtype, lines, ways, line_bytes, window, threshold)
    finally:
        for k, v in old_env.items():
            if v is None:
                del os.environ[k]
            else:
                os.environ[k] = v
    buffered = bool(window or push_depth0)
    with ses_cm as ses:
        ses.store_view()[:] = feats_u8
        if hot is not None and len(hot):
            ses.pin_hot(hot)
        if policy is not None:
            ses.set_policy(*policy)
        if rows_per_line != 1:
            ses.set_rows_per_line(rows_per_line)
        if threshold and accum_mode:
            ses.set_accum_mode(accum_mode)
        if dedup:
            ses.set_group_dedup(True)                         # one transfer per CPU-buffer row and group
        dev = [ses.to_device(b) for b in batches]
        torch.cuda.synchronize()
        push_stream = torch.cuda.Stream() if two_streams else None
        outs, uniqs, invs, seqs = [], [], [], []
        pushed = 0
        for t, raw in enumerate(batches):
            while buffered and pushed < len(batches) and pushed <= t + window:
                ses.push(dev[pushed], stream=push_stream)
                pushed += 1
            cap = max(len(raw), 1)
            out = torch.full((cap, row_bytes), 0xA5, dtype=torch.uint8, device="cuda")
            uq = torch.full((cap,), -7, dtype=ses.torch_id, device="cuda")
            inv = torch.full((cap,), -1, dtype=torch.int32, device="cuda") if with_inverse else None
            ids_arg = None if (use_head and buffered) else dev[t]
            seqs.append(ses.gather(ids_arg, out, uq, inv if ids_arg is not None else None))
            outs.append(out); uniqs.append(uq); invs.append(inv if ids_arg is not None else None)
        ses.flush()
        torch.cuda.synchronize()
        seen_hot = set()                                      # CPU-buffer rows the open group already fetches
        for t, raw in enumerate(batches):
            want_u, want_rows, want_stats = want[t]
            st = ses.stats(seqs[t])
            assert st.status == 0
            if dedup and hot is not None and len(hot):
                mine = set(np.intersect1d(want_u, hot).tolist())
                assert st.n_cpu_again == len(mine & seen_hot), (label, t, st.n_cpu_again, len(mine & seen_hot))
                seen_hot = set() if accum[t][1] else seen_hot | mine      # (the oracle's groups: closed by this gather?)
            else:
                assert st.n_cpu_again == 0
            assert st.as_tuple() == tuple(int(x) for x in want_stats), (label, t, st.as_tuple(), want_stats.tolist())
            assert st.n_line_fills == line_fills[t], (label, t, st.n_line_fills, line_fills[t])
            m = len(want_u)
            got_u = uniqs[t][:m].cpu().numpy()
            np.testing.assert_array_equal(got_u, want_u.astype(got_u.dtype), err_msg=f"{label} batch {t} unique")
            got_rows = outs[t][:m].cpu().numpy()
            assert np.array_equal(got_rows, want_rows), f"{label} batch {t}: gathered rows differ"
            if m < outs[t].shape[0]:                          # nothing written past the distinct count
                assert bool((outs[t][m:] == 0xA5).all())
            if invs[t] is not None:
                inv = invs[t][:len(raw)].cpu().numpy()
                np.testing.assert_array_equal(want_u[inv], np.asarray(raw, dtype=np.int64))
            # the accumulator's own behaviour: rows still queued after this gather, and whether it closed its group
            assert (st.n_pending, st.flushed) == accum[t][:2], (label, t, st.n_pending, st.flushed, accum[t])
        if check_state:
            tags, stamps = ses.snapshot()
            np.testing.assert_array_equal(tags, sim.tags, err_msg=f"{label} tags")
            np.testing.assert_array_equal(stamps, sim.stamps, err_msg=f"{label} stamps")


def zipf_batches(rng, n, n_batches, size, a=1.3):
    return [np.minimum(rng.zipf(a, size=int(rng.integers(size // 2, size + 1))) - 1, n - 1).astype(np.int64)
            for _ in range(n_batches)]


def rand_feats(rng, n, row_bytes):
    return rng.integers(0, 256, size=(n, row_bytes), dtype=np.uint8)


# ------------------------------------------------------------------ configs

def test_tiny_config_full_parity(gpu, oracle_mod):
    cfg = CONFIGS["tiny"]
    g = wl.make_graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max)
    table = wl.normal_table(np.float32)
    feats = wl.feature_rows(cfg.seed, np.arange(cfg.n_nodes), cfg.dim, table)
    hot = wl.hot_nodes(g, cfg.cpu_rows)
    batches = [wl.sample_minibatch(g, cfg.seed, b, cfg.fanouts, cfg.n_seeds) for b in range(cfg.n_batches)]
    run_case(gpu, oracle_mod, feats, batches, id_dtype=np.int32, lines=cfg.cache_lines, ways=cfg.ways,
             line_bytes=cfg.line_bytes, window=cfg.window, hot=hot, with_inverse=True, label="tiny")
    run_case(gpu, oracle_mod, feats, batches, id_dtype=np.int32, lines=cfg.cache_lines, ways=cfg.ways,
             line_bytes=cfg.line_bytes, window=cfg.window, hot=hot, use_head=True, label="tiny/head")


@pytest.mark.parametrize("pipeline", ["0", "1"])
@pytest.mark.parametrize("window,use_head", [(4, True), (4, False), (1, True), (12, True), (0, True)])
def test_pushes_on_their_own_stream(gpu, oracle_mod, window, use_head, pipeline):
    """The documented way to overlap classification with row movement: window
    pushes on one stream, gathers on another, many minibatches in flight."""
    rng = np.random.default_rng(77 + window)
    n = 40_000
    feats = rand_feats(rng, n, 1024)
    batches = zipf_batches(rng, n, 40, 6000, a=1.12)
    run_case(gpu, oracle_mod, feats, batches, id_dtype=np.int64, lines=4096, ways=8, line_bytes=1024, window=window,
             hot=rng.choice(n, 800, replace=False), use_head=use_head, two_streams=True, pipeline=pipeline,
             push_depth0=True, label=f"2streams/W{window}/pipe{pipeline}")


def test_two_streams_without_the_internal_stream(gpu, oracle_mod):
    """Small caches and accumulating caches run every kernel on the stream of the
    call; calls that alternate between two streams must still be ordered."""
    rng = np.random.default_rng(5150)
    n = 8000
    feats = rand_feats(rng, n, 256)
    batches = zipf_batches(rng, n, 24, 1500, a=1.15)
    for threshold in (0, 500):
        run_case(gpu, oracle_mod, feats, batches, id_dtype=np.int32, lines=512, ways=4, line_bytes=256, window=3,
                 threshold=threshold, hot=rng.choice(n, 100, replace=False), use_head=True, two_streams=True,
                 label=f"2streams-small/thr{threshold}")


def test_tiny_config_oracle_generated_inputs(gpu, oracle_mod):
    """End to end from the seed with the oracle's own generator and sampler."""
    cfg = CONFIGS["tiny"]
    g = oracle_mod.Graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max)
    table = wl.normal_table(np.float32)
    feats = oracle_mod.feat_rows(cfg.seed, np.arange(cfg.n_nodes), cfg.dim, table)
    batches = [g.sample(cfg.seed, b, cfg.fanouts, cfg.n_seeds) for b in range(cfg.n_batches)]
    run_case(gpu, oracle_mod, feats, batches, id_dtype=np.int32, lines=cfg.cache_lines, ways=cfg.ways,
             line_bytes=cfg.line_bytes, window=cfg.window, hot=g.hot_nodes(cfg.cpu_rows), label="tiny/oracle-inputs")


def test_medium_config_first_batches(gpu, oracle_mod):
    cfg = CONFIGS["medium"]
    n = 200_000                                               # one fifth of the node count, every ratio kept
    c = wl.scaled(cfg, n)
    g = wl.make_graph(c.seed, n, c.ell, c.p4, min(n - 1, 65535))
    table = wl.normal_table(np.float16)
    feats = np.empty((n, c.dim), dtype=np.float16)
    wl.fill_store(c.seed, n, c.dim, table, feats)
    hot = wl.hot_nodes(g, c.cpu_rows)
    batches = [wl.sample_minibatch(g, c.seed, b, c.fanouts, c.n_seeds) for b in range(24)]
    run_case(gpu, oracle_mod, feats, batches, id_dtype=np.int64, lines=c.cache_lines, ways=c.ways,
             line_bytes=c.line_bytes, window=c.window, hot=hot, label="medium/5")


# ------------------------------------------------------- shapes and policies

@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("ways", [1, 2, 4, 8, 16, 64])
def test_associativity_sweep(gpu, oracle_mod, ways, fused):
    rng = np.random.default_rng(100 + ways)
    n = 3000
    feats = rand_feats(rng, n, 256)
    lines = ways * 37                                          # 37 sets: not a power of two
    run_case(gpu, oracle_mod, feats, zipf_batches(rng, n, 14, 700, a=1.2), id_dtype=np.int64, lines=lines, ways=ways,
             line_bytes=256, window=2, hot=rng.choice(n, 50, replace=False), fused=fused, label=f"ways{ways}/fused{fused}")


@pytest.mark.parametrize("window", [0, 1, 3, 9])
@pytest.mark.parametrize("id_dtype", [np.int32, np.int64])
def test_window_depths_and_id_widths(gpu, oracle_mod, window, id_dtype):
    rng = np.random.default_rng(7 * window + np.dtype(id_dtype).itemsize)
    n = 5000
    feats = rand_feats(rng, n, 512)
    run_case(gpu, oracle_mod, feats, zipf_batches(rng, n, 16, 900, a=1.15), id_dtype=id_dtype, lines=512, ways=4,
             line_bytes=512, window=window, hot=rng.choice(n, 80, replace=False), label=f"W{window}")


@pytest.mark.parametrize("row_bytes,line_bytes", [(16, 16), (64, 128), (528, 1024), (2048, 2048), (3072, 4096), (4096, 4096)])
def test_row_and_line_sizes(gpu, oracle_mod, row_bytes, line_bytes):
    rng = np.random.default_rng(row_bytes)
    n = 2000
    feats = rand_feats(rng, n, row_bytes)
    run_case(gpu, oracle_mod, feats, zipf_batches(rng, n, 10, 600, a=1.25), id_dtype=np.int64, lines=256, ways=8,
             line_bytes=line_bytes, window=2, hot=rng.choice(n, 30, replace=False), label=f"R{row_bytes}")


def test_many_ids_per_set_needs_multiword_miss_mask(gpu, oracle_mod):
    """A small cache over a long table: more than 64 IDs share a set."""
    rng = np.random.default_rng(11)
    n = 20_000
    feats = rand_feats(rng, n, 64)
    batches = [rng.integers(0, n, size=5000) for _ in range(8)]        # ~20 % of all IDs per minibatch: heavy bypass
    for fused in (True, False):
        run_case(gpu, oracle_mod, feats, batches, id_dtype=np.int64, lines=4 * 50, ways=4, line_bytes=64, window=1,
                 fused=fused, label=f"multiword/fused{fused}")


def test_cache_as_large_as_store_all_hits_after_warmup(gpu, oracle_mod):
    rng = np.random.default_rng(12)
    n, ways, n_sets = 4096, 16, 256
    feats = rand_feats(rng, n, 768)
    batches = [rng.integers(0, n, size=6000) for _ in range(12)] + [np.arange(n)] * 2
    run_case(gpu, oracle_mod, feats, batches, id_dtype=np.int64, lines=ways * n_sets, ways=ways, line_bytes=1024,
             window=3, label="resident")


def test_degenerate_inputs(gpu, oracle_mod):
    rng = np.random.default_rng(13)
    n = 1000
    feats = rand_feats(rng, n, 128)
    batches = [np.array([], dtype=np.int64), np.array([n - 1]), np.full(5000, 17), np.arange(n), np.array([0, n - 1, 0]),
               np.array([], dtype=np.int64), rng.integers(0, n, 257), rng.integers(0, n, 2049)]
    for window in (0, 2):
        run_case(gpu, oracle_mod, feats, batches, id_dtype=np.int32, lines=64, ways=4, line_bytes=128, window=window,
                 hot=np.array([0, 17, n - 1]), with_inverse=True, label=f"degenerate/W{window}")


def test_long_raw_list_many_tiles(gpu, oracle_mod):
    """Raw lists spanning many workgroup tiles with heavy repetition (hub nodes)."""
    rng = np.random.default_rng(14)
    n = 300_000
    feats = rand_feats(rng, n, 64)
    batches = [np.minimum(rng.zipf(1.1, size=700_001) - 1, n - 1) for _ in range(3)]
    for fused in (False, True):
        run_case(gpu, oracle_mod, feats, batches, id_dtype=np.int64, lines=8 * 1024, ways=8, line_bytes=64, window=1,
                 hot=np.arange(0, 2000, 3), with_inverse=True, fused=fused, label=f"long/fused{fused}")


# ---------------------------------------------------------------- accumulator

@pytest.mark.parametrize("pipeline", ["0", "1"])
@pytest.mark.parametrize("threshold,mode", [(1, 0), (300, 0), (2000, 0), (100_000, 0), (150, 1), (40, 1)])
@pytest.mark.parametrize("window", [0, 3])
def test_accumulator_changes_nothing(gpu, oracle_mod, threshold, mode, window, pipeline):
    """Section 3.2: merging the accesses of consecutive minibatches is a scheduling
    choice; counters and tensors are those of the unmerged run, and the groups
    (rows pending after each gather, which gather closes a group) are the oracle's,
    for a fixed threshold and for one that follows the redirected share."""
    rng = np.random.default_rng(1000 + threshold + window)
    n = 6000
    feats = rand_feats(rng, n, 256)
    run_case(gpu, oracle_mod, feats, zipf_batches(rng, n, 60, 400, a=1.2), id_dtype=np.int64, lines=128, ways=4,
             line_bytes=256, window=window, threshold=threshold, accum_mode=mode, hot=rng.choice(n, 60, replace=False),
             pipeline=pipeline, two_streams=pipeline == "1", use_head=bool(window), fused=bool(threshold % 7 % 2),
             label=f"accum{threshold}/mode{mode}/W{window}/pipe{pipeline}")


@pytest.mark.parametrize("pipeline", ["0", "1"])
def test_accumulator_lines_reused_inside_a_group(gpu, oracle_mod, pipeline):
    """A cache of a few lines under long groups: lines are hit, evicted and refilled several times before
    their group moves (copies out of a line that is refilled later in the group, hits on lines whose fill
    is still queued, lines installed twice in one group)."""
    rng = np.random.default_rng(31337)
    n, R = 300, 64
    feats = rand_feats(rng, n, R)
    batches = [rng.integers(0, 40, size=int(rng.integers(3, 25))) for _ in range(60)]   # 40 hot IDs over 8 lines
    for threshold in (60, 200, 10_000):
        run_case(gpu, oracle_mod, feats, batches, id_dtype=np.int32, lines=8, ways=2, line_bytes=R, window=0,
                 threshold=threshold, pipeline=pipeline, fused=False, label=f"accum-reuse/thr{threshold}/pipe{pipeline}")
        run_case(gpu, oracle_mod, feats, batches, id_dtype=np.int64, lines=8, ways=8, line_bytes=R, window=2,
                 threshold=threshold, pipeline=pipeline, hot=np.array([3, 17]), use_head=True, two_streams=True,
                 label=f"accum-reuse/W2/thr{threshold}/pipe{pipeline}")


@pytest.mark.parametrize("pipeline", ["0", "1"])
def test_accumulator_fetches_a_cpu_buffer_row_once_per_group(gpu, oracle_mod, pipeline):
    """gids_cache_set_group_dedup with single gathers: a CPU-buffer row that an earlier minibatch of the open group
    already fetches comes as a copy of that output row.  Outputs, counters, groups and cache state as without it;
    n_cpu_again equals its definition over the oracle's groups.  Fixed and adaptive thresholds, one launch or a
    kernel each for commit, queueing and counters."""
    rng = np.random.default_rng(4711)
    n, R = 6000, 128
    feats = rand_feats(rng, n, R)
    hot = rng.choice(n, 1500, replace=False)
    batches = [np.concatenate([rng.choice(hot, int(rng.integers(50, 400))), rng.integers(0, n, size=300)]).astype(np.int64)
               for _ in range(50)]
    batches[7] = np.array([], dtype=np.int64)
    for threshold, mode, fused in ((900, 0, True), (5000, 0, False), (2500, 1, True), (10**9, 0, True)):
        run_case(gpu, oracle_mod, feats, batches, id_dtype=np.int64, lines=64 * 4, ways=4, line_bytes=R, window=3,
                 threshold=threshold, accum_mode=mode, hot=hot, use_head=True, two_streams=True, pipeline=pipeline,
                 fused=fused, dedup=True, label=f"once-per-group/thr{threshold}/mode{mode}/pipe{pipeline}")


def test_accumulator_outputs_follow_the_callers_stream(gpu, oracle_mod):
    """With the library's internal stream on, an accumulating cache classifies ahead of the caller's stream.
    Whatever the caller still has queued on its stream for an output buffer (here: a slow kernel, then a fill
    of the distinct-ID buffer and of the rows) must happen before the library writes that buffer."""
    import os
    torch, gids, GatherSession = gpu
    rng = np.random.default_rng(99)
    n, R = 20_000, 256
    feats = rand_feats(rng, n, R)
    lists = zipf_batches(rng, n, 6, 3000, a=1.15)
    old = os.environ.get("GIDS_PIPELINE")
    os.environ["GIDS_PIPELINE"] = "1"
    try:
        ses = GatherSession(n, R, np.int64, 1024, 8, R, 2, 5000)
    finally:
        if old is None:
            del os.environ["GIDS_PIPELINE"]
        else:
            os.environ["GIDS_PIPELINE"] = old
    with ses:
        ses.store_view()[:] = feats
        dev = [ses.to_device(b) for b in lists]
        a = torch.randn(4096, 4096, device="cuda")
        ps = torch.cuda.Stream()
        got, pushed = [], 0
        for t, raw in enumerate(lists):
            while pushed < len(lists) and pushed <= t + 2:
                ses.push(dev[pushed], stream=ps)
                pushed += 1
            out = torch.empty((len(raw), R), dtype=torch.uint8, device="cuda")
            uq = torch.empty(len(raw), dtype=torch.int64, device="cuda")
            for _ in range(6):
                a = a @ a * 1e-4                                # a few milliseconds on the caller's stream ...
            out.fill_(0xA5)                                     # ... behind which the buffers are prepared
            uq.fill_(-7)
            ses.gather(None, out, uq)
            got.append((out, uq))
        ses.flush()
        torch.cuda.synchronize()
        for (out, uq), raw in zip(got, lists):
            u = np.unique(raw)
            assert np.array_equal(uq[:len(u)].cpu().numpy(), u)
            assert np.array_equal(out[:len(u)].cpu().numpy(), feats[u])


# ------------------------------------------------------------------- errors

def test_device_found_errors(gpu, oracle_mod):
    torch, gids, GatherSession = gpu
    feats = np.arange(100 * 64, dtype=np.uint8).reshape(100, 64)

    def fresh(window):
        s = GatherSession(100, 64, np.int64, 16, 4, 64, window)
        s.store_view()[:] = feats
        return s

    out = torch.zeros((8, 64), dtype=torch.uint8, device="cuda")
    # an ID outside the table
    with fresh(0) as s:
        seq = s.gather(s.to_device([1, 100]), out)
        with pytest.raises(gids.GidsError) as e:
            s.stats(seq)
        assert e.value.code == gids.GIDS_E_RANGE
        with pytest.raises(gids.GidsError) as e:                # sticky afterwards
            s.gather(s.to_device([1]), out)
        assert e.value.code == gids.GIDS_E_RANGE
    # the same while the inverse map is asked for: the bitmap is kept beyond the emit kernel and cleared through
    # the distinct-ID list, which therefore has to be written even for a list that fails
    with fresh(0) as s:
        inv = torch.zeros(8, dtype=torch.int32, device="cuda")
        uq = torch.zeros(8, dtype=torch.int64, device="cuda")
        seq = s.gather(s.to_device([1, 100, 5, 99, -3]), out, uq, inv)
        with pytest.raises(gids.GidsError) as e:
            s.stats(seq)
        assert e.value.code == gids.GIDS_E_RANGE
        assert bool((out == 0).all()) and bool((inv == 0).all())
        with pytest.raises(gids.GidsError) as e:                # sticky afterwards
            s.gather(s.to_device([1]), out)
        assert e.value.code == gids.GIDS_E_RANGE
    with fresh(1) as s:                                         # ... and a list that is not the window head
        inv = torch.zeros(8, dtype=torch.int32, device="cuda")
        s.push(s.to_device([1, 2]))
        seq = s.gather(s.to_device([3, 4, 3]), out, None, inv)
        with pytest.raises(gids.GidsError) as e:
            s.stats(seq)
        assert e.value.code == gids.GIDS_E_ORDER
        assert bool((out == 0).all())
    # a device error reaches a caller that never reads counters: the next call after the gather has finished
    with fresh(0) as s:
        s.gather(s.to_device([1, 100]), out)
        torch.cuda.synchronize()
        with pytest.raises(gids.GidsError) as e:
            s.flush()
        assert e.value.code == gids.GIDS_E_RANGE
    # more distinct IDs than output rows
    with fresh(0) as s:
        seq = s.gather(s.to_device(np.arange(9)), out)
        with pytest.raises(gids.GidsError) as e:
            s.stats(seq)
        assert e.value.code == gids.GIDS_E_SPACE
        assert bool((out == 0).all())
    # window protocol
    with fresh(1) as s:
        with pytest.raises(gids.GidsError) as e:
            s.gather(s.to_device([1]), out)
        assert e.value.code == gids.GIDS_E_ORDER                # nothing buffered
        s.push(s.to_device([1, 2]))
        s.push(s.to_device([3]))
        with pytest.raises(gids.GidsError) as e:
            s.push(s.to_device([4]))
        assert e.value.code == gids.GIDS_E_FULL
        seq = s.gather(s.to_device([3]), out)                   # not the head
        with pytest.raises(gids.GidsError) as e:
            s.stats(seq)
        assert e.value.code == gids.GIDS_E_ORDER
        assert bool((out == 0).all())
    with fresh(0) as s:                                         # depth 0 buffers one list, the next gather's
        s.push(s.to_device([1]))
        with pytest.raises(gids.GidsError) as e:
            s.push(s.to_device([2]))
        assert e.value.code == gids.GIDS_E_FULL
        seq = s.gather(None, out)
        assert s.stats(seq).n_unique == 1


@pytest.mark.parametrize("window,ways", [(0, 4), (3, 8), (0, 64), (2, 1), (1, 16)])
def test_random_base_policy(gpu, oracle_mod, window, ways):
    """The paper's base policy (random eviction), seeded: same victims as the oracle."""
    rng = np.random.default_rng(4242 + window + ways)
    n = 6000
    feats = rand_feats(rng, n, 128)
    for seed in (0, 0xDEADBEEF12345):
        run_case(gpu, oracle_mod, feats, zipf_batches(rng, n, 25, 700, a=1.15), id_dtype=np.int64, lines=ways * 13,
                 ways=ways, line_bytes=128, window=window, hot=rng.choice(n, 40, replace=False),
                 policy=(1, seed), fused=seed == 0, label=f"random-policy/W{window}/ways{ways}")


# ------------------------------------------------------------- randomised

@pytest.mark.parametrize("case", range(48))
def test_random_configurations(gpu, oracle_mod, case):
    """Seeded random geometry, window, accumulator threshold, stream use and
    list shapes (the draw is printed, so a failure names its case)."""
    rng = np.random.default_rng(9000 + case)
    n = int(rng.choice([63, 64, 65, 1000, 4097, 30_011]))
    ways = int(rng.choice([1, 2, 4, 8, 16, 32]))
    n_sets = int(rng.integers(1, max(2, n // (ways * int(rng.integers(1, 80))) + 2)))
    row_bytes = int(rng.choice([16, 48, 256, 1040, 2048]))
    line_bytes = row_bytes + 16 * int(rng.integers(0, 3))
    window = int(rng.choice([0, 0, 1, 2, 5, 11]))
    threshold = int(rng.choice([0, 0, 0, 7, 900]))
    accum_mode = int(case % 2) if threshold else 0
    id_dtype = np.int32 if rng.random() < 0.5 else np.int64
    n_hot = int(rng.integers(0, max(1, n // 10)))
    size = int(rng.integers(1, 4 * n))
    a = float(rng.choice([1.05, 1.3, 2.0]))
    batches = []
    for _ in range(int(rng.integers(3, 22))):
        m = int(rng.integers(0, size + 1))
        if rng.random() < 0.5:
            b = np.minimum(rng.zipf(a, size=m) - 1, n - 1)
        else:
            b = rng.integers(0, n, size=m)
        batches.append(b.astype(np.int64))
    feats = rand_feats(rng, n, row_bytes)
    # the second half of the cases also draws the stream arrangement inside the library and pushes at depth 0
    extra = {}
    if case >= 24:
        extra = dict(pipeline=str(int(rng.integers(0, 2))), push_depth0=bool(rng.random() < 0.5),
                     wide_index=bool(rng.random() < 0.5))
        if extra["push_depth0"] and window == 0 and rng.random() < 0.5:
            extra["use_head_override"] = True
    use_head_override = extra.pop("use_head_override", False)
    extra["fused"] = [None, True, False][case % 3]
    run_case(gpu, oracle_mod, feats, batches, id_dtype=id_dtype, lines=ways * n_sets, ways=ways, line_bytes=line_bytes,
             window=window, threshold=threshold, accum_mode=accum_mode,
             hot=rng.choice(n, n_hot, replace=False) if n_hot else None,
             use_head=bool(use_head_override or (window and rng.random() < 0.5)), with_inverse=bool(rng.random() < 0.5),
             two_streams=bool(rng.random() < 0.5), policy=(1, case) if rng.random() < 0.3 else None,
             dedup=bool(threshold and case % 2 == 0), label=f"random{case}", **extra)


def test_link_calibration_is_sane(gpu):
    """Eq. 2-3's inputs measured on the box: a rate of the order of the PCIe link and a small fixed overhead."""
    torch, gids, GatherSession = gpu
    store = gids.gids_store_create(2_000_000, 2048, 8)         # 4 GB: larger than any on-chip cache
    try:
        rate, overhead = gids.gids_store_calibrate(store)
        gbs = rate * 2048 / 1e9
        assert 5.0 < gbs < 70.0, gbs                            # a PCIe Gen3 x16 ... Gen5 x16 link
        assert -50e-6 < overhead < 500e-6, overhead
        n95 = gids.gids_accum_threshold(rate, max(overhead, 1e-6), 0.0, 0.95)
        assert 10 < n95 < 1e6
    finally:
        gids.gids_store_destroy(store)


def test_layerwise_id_streams(gpu, oracle_mod):
    """The second sampler shape (Section 4.7): fixed-size layers drawn by connection count give
    lists with much heavier overlap between minibatches than neighbourhood sampling."""
    cfg = CONFIGS["tiny"]
    g = wl.make_graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max)
    table = wl.normal_table(np.float32)
    feats = wl.feature_rows(cfg.seed, np.arange(cfg.n_nodes), cfg.dim, table)
    hot = wl.hot_nodes(g, cfg.cpu_rows)
    batches = [wl.layerwise_minibatch(g, cfg.seed, b, (512, 512), cfg.n_seeds) for b in range(cfg.n_batches)]
    for window in (0, cfg.window):
        run_case(gpu, oracle_mod, feats, batches, id_dtype=np.int32, lines=cfg.cache_lines, ways=cfg.ways,
                 line_bytes=cfg.line_bytes, window=window, hot=hot, label=f"layerwise/W{window}")
        run_case(gpu, oracle_mod, feats, batches, id_dtype=np.int32, lines=cfg.cache_lines, ways=cfg.ways,
                 line_bytes=cfg.line_bytes, window=window, label=f"layerwise/nohot/W{window}", policy=(1, 9))


def test_two_caches_share_one_store(gpu, oracle_mod):
    """Several caches may read one store: two of different shape and policy, calls interleaved on two
    streams, each equal to its own oracle run."""
    torch, gids, GatherSession = gpu
    rng = np.random.default_rng(4242)
    n, R = 30_000, 512
    feats = rand_feats(rng, n, R)
    lists = [zipf_batches(rng, n, 16, 4000, a=1.15) for _ in range(2)]
    shapes = [dict(lines=2048, ways=8, window=3, policy=None), dict(lines=1024, ways=4, window=0, policy=(1, 5))]
    want = []
    for sh, batches in zip(shapes, lists):
        sim = oracle_mod.Sim(n, sh["lines"], sh["ways"], sh["window"], R, R, feats)
        if sh["policy"]:
            sim.set_policy(*sh["policy"])
        res, pushed = [], 0
        for t, raw in enumerate(batches):
            while sh["window"] and pushed < len(batches) and pushed <= t + sh["window"]:
                sim.push(batches[pushed])
                pushed += 1
            res.append(sim.gather(raw))
        want.append((res, sim))
    store = gids.gids_store_create(n, R, 8)
    try:
        ses = [GatherSession(n, R, np.int64, sh["lines"], sh["ways"], R, sh["window"], store_handle=store)
               for sh in shapes]
        ses[0].store_view()[:] = feats
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        for s, sh in zip(ses, shapes):
            if sh["policy"]:
                s.set_policy(*sh["policy"])
        dev = [[s.to_device(b) for b in batches] for s, batches in zip(ses, lists)]
        torch.cuda.synchronize()
        outs = [[], []]
        pushed = [0, 0]
        for t in range(16):
            for k in (0, 1):                                  # alternate between the two caches
                w = shapes[k]["window"]
                while w and pushed[k] < 16 and pushed[k] <= t + w:
                    ses[k].push(dev[k][pushed[k]], stream=streams[k])
                    pushed[k] += 1
                cap = len(lists[k][t])
                out = torch.empty((cap, R), dtype=torch.uint8, device="cuda")
                uq = torch.empty(cap, dtype=torch.int64, device="cuda")
                seq = ses[k].gather(None if w else dev[k][t], out, uq, stream=streams[k])
                outs[k].append((seq, out, uq))
        torch.cuda.synchronize()
        for k in (0, 1):
            res, sim = want[k]
            for t, (seq, out, uq) in enumerate(outs[k]):
                u, rows, stats = res[t]
                assert ses[k].stats(seq).as_tuple() == tuple(int(x) for x in stats), (k, t)
                assert np.array_equal(uq[:len(u)].cpu().numpy(), u)
                assert np.array_equal(out[:len(u)].cpu().numpy(), rows), (k, t)
            tags, stamps = ses[k].snapshot()
            assert np.array_equal(tags, sim.tags) and np.array_equal(stamps, sim.stamps)
        for s in ses:
            s.close()
    finally:
        gids.gids_store_destroy(store)


@pytest.mark.parametrize("two_streams", [False, True])
def test_depth_zero_with_lists_pushed_ahead(gpu, oracle_mod, two_streams):
    """At window depth 0 one list may be pushed before its gather so that its deduplication runs ahead; nothing
    is pinned, so counters, rows and final tags equal the oracle's depth-0 run (plain LRU), whether a gather
    takes the pushed list, repeats it as an argument, or comes without a push at all."""
    torch, gids, GatherSession = gpu
    rng = np.random.default_rng(606)
    n, R = 50_000, 1024
    feats = rand_feats(rng, n, R)
    batches = zipf_batches(rng, n, 30, 5000, a=1.12)
    hot = rng.choice(n, 600, replace=False)
    sim = oracle_mod.Sim(n, 4096, 8, 0, R, R, feats)
    sim.set_hot(hot)
    want = [sim.gather(raw) for raw in batches]
    with GatherSession(n, R, np.int64, 4096, 8, R, 0) as ses:      # 4 MiB cache: single-stream mode ...
        ses.store_view()[:] = feats
        ses.pin_hot(hot)
        check_depth_zero(torch, ses, batches, want, sim, two_streams)
    sim = oracle_mod.Sim(n, 65536, 8, 0, R, R, feats)
    sim.set_hot(hot)
    want = [sim.gather(raw) for raw in batches]
    with GatherSession(n, R, np.int64, 65536, 8, R, 0) as ses:     # ... 64 MiB: the internal stream is used
        ses.store_view()[:] = feats
        ses.pin_hot(hot)
        check_depth_zero(torch, ses, batches, want, sim, two_streams)


def check_depth_zero(torch, ses, batches, want, sim, two_streams):
    dev = [ses.to_device(b) for b in batches]
    torch.cuda.synchronize()
    ps = torch.cuda.Stream() if two_streams else None
    got = []
    for t, raw in enumerate(batches):
        mode = t % 3                                            # 0: push + gather(None), 1: push + gather(ids), 2: no push
        if mode != 2:
            ses.push(dev[t], stream=ps)
        out = torch.full((len(raw), ses.row_bytes), 0x5A, dtype=torch.uint8, device="cuda")
        uq = torch.empty(len(raw), dtype=torch.int64, device="cuda")
        got.append((ses.gather(None if mode == 0 else dev[t], out, uq), out, uq))
    torch.cuda.synchronize()
    for t, (seq, out, uq) in enumerate(got):
        u, rows, stats = want[t]
        assert ses.stats(seq).as_tuple() == tuple(int(x) for x in stats), t
        assert np.array_equal(uq[:len(u)].cpu().numpy(), u)
        assert np.array_equal(out[:len(u)].cpu().numpy(), rows), t
    tags, stamps = ses.snapshot()
    assert np.array_equal(tags, sim.tags) and np.array_equal(stamps, sim.stamps)


@pytest.mark.parametrize("rows,window,policy,id_dtype", [(8, 3, None, np.int64), (2, 0, None, np.int32), (4, 5, (1, 3), np.int64),
                                                          (3, 2, None, np.int64), (16, 1, None, np.int32)])
def test_several_rows_per_cache_line(gpu, oracle_mod, rows, window, policy, id_dtype):
    """Lines of several node rows (the 4 KB cache-lines of Section 3.3 under 512 B rows): counters, the number of
    lines filled, every gathered row and the final tags (store line numbers) equal the oracle's."""
    rng = np.random.default_rng(300 + rows)
    n, R = 20_011, 64                                          # the table's last line is partial
    feats = rand_feats(rng, n, R)
    # neighbourhoods of hubs: many requested rows share a line
    batches = []
    for _ in range(18):
        hubs = np.minimum(rng.zipf(1.2, size=600) - 1, n - 1)
        near = np.clip(hubs + rng.integers(-6, 7, size=600), 0, n - 1)
        batches.append(np.concatenate([hubs, near, rng.integers(0, n, size=200)]).astype(np.int64))
    ways = 4
    for pipeline in ("0", "1"):
        run_case(gpu, oracle_mod, feats, batches, id_dtype=id_dtype, lines=ways * 61, ways=ways, line_bytes=rows * R + 16,
                 window=window, hot=rng.choice(n, 150, replace=False), policy=policy, rows_per_line=rows,
                 use_head=bool(window), two_streams=True, pipeline=pipeline, label=f"rows{rows}/W{window}/pipe{pipeline}")
    # a line for every store line: after one row of each, nothing misses
    lines = ((n + rows - 1) // rows + ways - 1) // ways * ways
    cover = [np.arange(0, n, rows), np.arange(n), rng.integers(0, n, size=3000)]
    run_case(gpu, oracle_mod, feats, cover, id_dtype=id_dtype, lines=lines, ways=ways, line_bytes=rows * R, window=0,
             rows_per_line=rows, label=f"rows{rows}/resident")


def test_rows_per_line_argument_checks(gpu):
    torch, gids, GatherSession = gpu
    with GatherSession(100, 64, np.int64, 16, 4, 256, 0) as s:
        with pytest.raises(gids.GidsError):
            s.set_rows_per_line(5)                             # 5 x 64 B do not fit a 256 B line
        with pytest.raises(gids.GidsError):
            s.set_rows_per_line(0)
        s.set_rows_per_line(4)
        out = torch.zeros((4, 64), dtype=torch.uint8, device="cuda")
        s.gather(s.to_device([1]), out)
        with pytest.raises(gids.GidsError):
            s.set_rows_per_line(2)                             # only before the first gather
    with GatherSession(100, 64, np.int64, 16, 4, 256, 0, 50) as s:
        with pytest.raises(gids.GidsError):
            s.set_rows_per_line(4)                             # not with the accumulator


@pytest.mark.parametrize("pipeline,threshold", [("0", 0), ("1", 0), ("0", 2500), ("1", 2500)])
def test_a_thousand_minibatches(gpu, oracle_mod, pipeline, threshold):
    """A long run on a small cache: the 64-entry rings of events and counters wrap many times, every slot of
    the window is reused hundreds of times; counters of every minibatch (read with a lag, as a training loop
    would), sampled tensors and the final tags must still equal the oracle's."""
    import os
    torch, gids, GatherSession = gpu
    cfg = CONFIGS["tiny"]
    g = wl.make_graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max)
    table = wl.normal_table(np.float32)
    feats = wl.feature_rows(cfg.seed, np.arange(cfg.n_nodes), cfg.dim, table).view(np.uint8).reshape(cfg.n_nodes, -1)
    hot = wl.hot_nodes(g, cfg.cpu_rows)
    base = [wl.sample_minibatch(g, cfg.seed, b, cfg.fanouts, cfg.n_seeds) for b in range(37)]
    n_b, W = 1000, 5
    lists = [base[(7 * t) % 37] for t in range(n_b)]
    sim = oracle_mod.Sim(cfg.n_nodes, cfg.cache_lines, cfg.ways, W, cfg.row_bytes, cfg.line_bytes, feats)
    sim.set_hot(hot)
    want, pushed = [], 0
    check_rows = set(range(0, n_b, 97)) | {n_b - 1}
    for t in range(n_b):
        while pushed < n_b and pushed <= t + W:
            sim.push(lists[pushed])
            pushed += 1
        want.append(sim.gather(lists[t], want_rows=t in check_rows))
    old = os.environ.get("GIDS_PIPELINE")
    os.environ["GIDS_PIPELINE"] = pipeline
    try:
        ses = GatherSession(cfg.n_nodes, cfg.row_bytes, np.int32, cfg.cache_lines, cfg.ways, cfg.line_bytes, W,
                            threshold)
    finally:
        if old is None:
            del os.environ["GIDS_PIPELINE"]
        else:
            os.environ["GIDS_PIPELINE"] = old
    with ses:
        ses.store_view()[:] = feats
        ses.pin_hot(hot)
        dev = [ses.to_device(b) for b in base]
        cap = max(len(b) for b in base)
        ses.reserve(cap)
        ps = torch.cuda.Stream()
        # with the accumulator an output must stay untouched until the flush that completes it
        n_ring = 16 if threshold else 3
        ring = [torch.empty((cap, cfg.row_bytes), dtype=torch.uint8, device="cuda") for _ in range(n_ring)]
        uq = torch.empty(cap, dtype=torch.int32, device="cuda")
        kept, seqs, pushed = {}, [], 0
        for t in range(n_b):
            while pushed < n_b and pushed <= t + W:
                ses.push(dev[(7 * pushed) % 37], stream=ps)
                pushed += 1
            if t in check_rows:
                kept[t] = (torch.empty((cap, cfg.row_bytes), dtype=torch.uint8, device="cuda"),
                           torch.empty(cap, dtype=torch.int32, device="cuda"))
                seqs.append(ses.gather(None, *kept[t]))
            else:
                seqs.append(ses.gather(None, ring[t % n_ring], uq))
            if threshold and t % n_ring == n_ring - 2:
                ses.flush()
            if t >= 30:
                k = t - 30
                assert ses.stats(seqs[k]).as_tuple() == tuple(int(x) for x in want[k][2]), k
        ses.flush()
        torch.cuda.synchronize()
        for k in range(n_b - 30, n_b):
            assert ses.stats(seqs[k]).as_tuple() == tuple(int(x) for x in want[k][2]), k
        for t, (out, u_dev) in kept.items():
            u, rows, _ = want[t]
            assert np.array_equal(u_dev[:len(u)].cpu().numpy(), u.astype(np.int32))
            assert np.array_equal(out[:len(u)].cpu().numpy(), rows), t
        tags, stamps = ses.snapshot()
        assert np.array_equal(tags, sim.tags) and np.array_equal(stamps, sim.stamps)
