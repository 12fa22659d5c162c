"""gids_gather_static, the gather that allocates nothing (its per-minibatch
buffers live in a fixed array inside the library), against gids_gather on the
same inputs: two caches of one shape over one store, one driven through each
entry point, must agree on every output and on the cache's final state."""
import numpy as np
import pytest

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


def lists(rng, n, sizes):
    return [np.minimum(rng.zipf(1.15, size=m) - 1, n - 1).astype(np.int64) for m in sizes]


@pytest.mark.parametrize("lines,window", [(65536, 3), (2048, 0)])   # 64 MiB: the library's internal stream is on; 2 MiB: off
def test_static_gather_equals_gather(gpu, lines, window):
    torch, gids, GatherSession = gpu
    rng = np.random.default_rng(2024 + window)
    n, R = 60_000, 1024
    feats = rng.integers(0, 256, size=(n, R), dtype=np.uint8)
    # two calls in a row, the second with a smaller input; then a few more of mixed sizes
    batches = lists(rng, n, [9000, 700, 5000, 1, 12000, 0, 3000, 8000])
    hot = rng.choice(n, 900, replace=False)
    store = gids.gids_store_create(n, R, 8)
    try:
        ref = GatherSession(n, R, np.int64, lines, 8, R, window, store_handle=store)
        sta = GatherSession(n, R, np.int64, lines, 8, R, window, store_handle=store)
        ref.store_view()[:] = feats
        results = []
        for ses, static in ((ref, False), (sta, True)):
            ses.pin_hot(hot)
            ses.reserve(max(len(b) for b in batches))          # the window's slots: a push never allocates after this
            dev = [ses.to_device(b) for b in batches]
            torch.cuda.synchronize()
            got, pushed = [], 0
            for t, raw in enumerate(batches):
                while window and pushed < len(batches) and pushed <= t + window:
                    ses.push(dev[pushed])
                    pushed += 1
                cap = max(len(raw), 1)
                out = torch.full((cap, R), 0xA5, dtype=torch.uint8, device="cuda")
                uq = torch.full((cap,), -7, dtype=torch.int64, device="cuda")
                ids = None if window else dev[t]
                seq = gids.gids_cache_gathers(ses.cache)
                stream = torch.cuda.current_stream().cuda_stream
                ptr = None if ids is None or not len(raw) else ids.data_ptr()
                print(f"[no-alloc] lines={lines} W={window} static={static} minibatch {t} raw={len(raw)}", flush=True)
                if static:
                    gids.gids_gather_static(ses.cache, ptr, 0 if ptr is None else len(raw), out.data_ptr(), cap,
                                            uq.data_ptr(), stream)
                else:
                    gids.gids_gather(ses.cache, ptr, 0 if ptr is None else len(raw), out.data_ptr(), cap, uq.data_ptr(),
                                     None, stream)
                got.append((seq, out, uq))
            torch.cuda.synchronize()                            # (also what lets the other cache use the array next)
            results.append(([(ses.stats(seq), out.cpu().numpy(), uq.cpu().numpy()) for seq, out, uq in got],
                            ses.snapshot()))
        (a, snap_a), (b, snap_b) = results
        for t, ((st_a, out_a, uq_a), (st_b, out_b, uq_b)) in enumerate(zip(a, b)):
            assert st_a.as_tuple() == st_b.as_tuple(), (t, st_a.as_tuple(), st_b.as_tuple())
            assert st_b.status == 0 and st_b.flushed == 1
            m = st_a.n_unique
            want_u = np.unique(batches[t])
            assert m == len(want_u)
            assert np.array_equal(uq_b[:m], want_u) and np.array_equal(uq_a, uq_b), t
            assert np.array_equal(out_a, out_b), t                  # rows and the untouched tail alike
            assert np.array_equal(out_b[:m], feats[want_u]), t      # ... and the plain definition
        assert np.array_equal(snap_a[0], snap_b[0]) and np.array_equal(snap_a[1], snap_b[1])
        ref.close()
        sta.close()
    finally:
        gids.gids_store_destroy(store)


def test_static_gather_limits(gpu):
    torch, gids, GatherSession = gpu
    out = torch.zeros((4, 64), dtype=torch.uint8, device="cuda")
    with GatherSession(100, 64, np.int64, 16, 4, 64, 0) as s:
        ids = torch.zeros(gids.GIDS_STATIC_MAX_IDS + 1, dtype=torch.int64, device="cuda")
        with pytest.raises(gids.GidsError) as e:                # beyond the static array: refused, nothing runs
            gids.gids_gather_static(s.cache, ids.data_ptr(), ids.numel(), out.data_ptr(), 4)
        assert e.value.code == gids.GIDS_E_INVAL
        assert gids.gids_cache_gathers(s.cache) == 0
        gids.gids_gather_static(s.cache, ids.data_ptr(), gids.GIDS_STATIC_MAX_IDS, out.data_ptr(), 4)   # the maximum
        st = s.stats(0)
        assert st.as_tuple() == (1, 0, 0, 1, 0)
    with GatherSession(100, 64, np.int64, 16, 4, 64, 0, 50) as s:  # an accumulating cache's queues grow on demand
        with pytest.raises(gids.GidsError) as e:
            gids.gids_gather_static(s.cache, None, 0, out.data_ptr(), 4)
        assert e.value.code == gids.GIDS_E_INVAL
    with GatherSession(100, 64, np.int64, 16, 4, 64, 2) as s:      # a buffered list longer than the array
        s.push(torch.zeros(gids.GIDS_STATIC_MAX_IDS + 1, dtype=torch.int64, device="cuda"))
        with pytest.raises(gids.GidsError) as e:
            gids.gids_gather_static(s.cache, None, 0, out.data_ptr(), 4)
        assert e.value.code == gids.GIDS_E_INVAL
