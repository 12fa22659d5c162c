#!/usr/bin/env python3
"""Benchmark of the minibatch feature gather on one MI355X.

One "step" = one pass of the whole hot path over one minibatch of synthetic
input: the gather of minibatch t (ID dedup/sort, window pop, CPU-buffer lookup,
tag probe, victim selection, line fills from the host store, hit scatter,
counters) plus the window push of minibatch t + W + 1 that keeps the look-ahead
full.  Sampling and graph generation are outside the timed region; every input
(raw ID lists, feature store) is resident before it starts (ID lists in HBM, the
store in pinned host memory, where the method keeps it).

Prints ONE JSON line: gathered GB/s (distinct IDs x row bytes / time), with the
hit/miss-weighted roofline (HBM peak for bytes that stay in HBM, host-link peak
for bytes that cross the link), the row mover's own roofline from HIP events on
the launch stream, and the CPU oracle timed on the machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
LINK_PEAK_GBS = 64.0         # PCIe Gen5 x16, nominal per direction (the box negotiates 32 GT/s x16)

# HBM / link traffic of the row mover per launch is a counter measurement (rocprofv3 --pmc, two runs) and cannot be
# taken inside this process; `roofline.traffic` is therefore null here, and `roofline.traffic_reference` names the
# committed counter summary of the same command on the same workload (other minibatches, another box) with the
# ratio of counted to algorithmic bytes found there.
TRAFFIC_REFERENCE = {
    "large": {"profile": "profiles/move_kernel_large_pmc.txt", "link_counted_over_algorithmic": 1.000,
              "hbm_write_counted_over_algorithmic": 1.00},
    "resident": {"profile": "profiles/move_kernel_resident_pmc.txt", "hbm_read_counted_over_algorithmic": 1.010,
                 "hbm_write_counted_over_algorithmic": 1.003},
}


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def pick_scale(cfg, wl, max_pinned_gib: float):
    """Largest node count whose store + CPU buffer fit the pinned-memory limit, ratios kept."""
    need = lambda c: (c.n_nodes * c.row_bytes + c.cpu_rows * c.row_bytes) / 2**30
    if need(cfg) <= max_pinned_gib:
        return cfg
    n = cfg.n_nodes
    while True:
        n = int(n * 0.9) // 1_000_000 * 1_000_000 if n > 2_000_000 else int(n * 0.9)
        c = wl.scaled(cfg, n)
        if need(c) <= max_pinned_gib:
            return c


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=12)
    ap.add_argument("--workload", default="large", choices=["tiny", "medium", "large", "resident", "skew"])
    ap.add_argument("--nodes", type=int, default=0, help="override the node count (ratios kept)")
    ap.add_argument("--max-pinned-gib", type=float, default=60.0,
                    help="pinned host memory the box grants one process (store + CPU buffer must fit)")
    ap.add_argument("--window", type=int, default=-1, help="override the window depth")
    ap.add_argument("--policy", default="lru", choices=["lru", "random"],
                    help="base replacement policy: LRU by minibatch, or the paper's seeded random eviction")
    ap.add_argument("--hot-by", default="indegree", choices=["indegree", "visits", "pagerank"],
                    help="what fills the CPU buffer: the nodes of highest in-degree (the configurations' rule), of "
                         "highest expected visits under the sampler (gids_graph_visit_scores), or of highest "
                         "weighted reverse PageRank (gids_graph_reverse_pagerank, the metric the paper names)")
    ap.add_argument("--layerwise", default="", metavar="S1,S2,..",
                    help="feed layer-wise sampled ID lists (the second sampler shape of Section 4.7): a fixed number "
                         "of nodes per layer, drawn by connection count, instead of neighbourhood sampling")
    ap.add_argument("--dim", type=int, default=0,
                    help="override the feature dimension (row bytes = dim x item size; lines shrink to the row, the "
                         "cache keeps its size in bytes), e.g. 256 for the 512 B rows of the paper's smaller datasets")
    ap.add_argument("--rows-per-line", type=int, default=1,
                    help="cache lines that hold this many consecutive node rows (line_bytes = rows x row_bytes, the "
                         "cache keeps its size in bytes): a miss brings the whole line in")
    ap.add_argument("--cache-lines", type=int, default=0, help="override the number of cache lines (rounded to ways)")
    ap.add_argument("--accum", type=int, default=0,
                    help="accumulator threshold in node accesses (raw list entries) per merged group of minibatches "
                         "(0 = every gather moves its own rows)")
    ap.add_argument("--group-dedup", action="store_true",
                    help="with --many: a CPU-buffer row that several steps of a call need crosses the link once "
                         "(gids_cache_set_group_dedup); the roofline fractions printed still charge every access one row")
    ap.add_argument("--many", type=int, default=0, metavar="K",
                    help="issue the steps K at a time through gids_gather_many (merged iterations: one call pushes K "
                         "lists and gathers K minibatches as one group); needs --accum > 0 for the group lists")
    ap.add_argument("--accum-adaptive", action="store_true",
                    help="read --accum as the store accesses wanted per launch (Eq. 2-3's N) and let the library "
                         "raise the node-access threshold by the redirected share (Section 3.2)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="time budget of the oracle leg")
    ap.add_argument("--pass-ids", action="store_true",
                    help="hand the raw ID list to gather again (it is then deduplicated a second time and checked "
                         "against the window head); default with a window: gather the buffered head list")
    ap.add_argument("--prewarm", type=int, default=-1,
                    help="before the warm-up minibatches, gather every node once in lists of this many consecutive "
                         "IDs (0 = off; default: on for the cache-resident workload, whose steady state is 'the "
                         "cache holds the whole store')")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain 1 GiB device copy three times (the known-size kernel that scales the "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    ap.add_argument("--probe-box", action="store_true",
                    help="measure the limits of this machine that the roofline arguments rest on (pinned host memory "
                         "a process is granted, the negotiated PCIe link, zero-copy and copy rates over it, device "
                         "copy rates, host cores and memory), print one JSON object and exit")
    ap.add_argument("--one-stream", action="store_true", help="issue pushes and gathers on the same stream")
    ap.add_argument("--sweep-skew", action="store_true",
                    help="run the skew sweep (seed Zipf s in {0, 0.8, 1.2} x window depth in {0, 4, 16}) on the "
                         "chosen workload's graph and store, one cache per point; prints one JSON object")
    ap.add_argument("--gpu-sampler", action="store_true",
                    help="produce every minibatch's ID list with the library's GPU neighbourhood sampler (graph in "
                         "HBM) inside the step, and push it without the host seeing it; also times the sampler alone")
    ap.add_argument("--sampler-zero-copy", action="store_true",
                    help="with --gpu-sampler: leave the CSR graph in pinned host memory and sample it zero-copy "
                         "(the paper's arrangement) instead of copying it to HBM")
    ap.add_argument("--consumer-ms", type=float, default=0.0,
                    help="third pass: a dummy consumer (bf16 matmuls of about this many ms per minibatch, on a "
                         "stream of its own) reads every gathered minibatch, to show how far the gather for "
                         "minibatch t + 1 overlaps the consumer of minibatch t (Section 3.2's pipeline)")
    ap.add_argument("--repeat", type=int, default=1,
                    help="run the workload this many times in one process, each with a cache of its own "
                         "(the last run is the one reported; the others are logged)")
    ap.add_argument("--others", default="auto", choices=["auto", "on", "off"],
                    help="append the other configurations (cache-resident, medium, tiny; 20 steps each) to the same JSON "
                         "line as `other_workloads`; auto: only when no option besides --gpus / --steps / --warmup is given")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the gather shards by minibatch, one cache per GPU; "
              "no multi-GPU path is built). Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch
    import workload as wl
    import paper_2306_16384_amd as gids
    from paper_2306_16384_amd.session import GatherSession

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the gather has no CPU path", file=sys.stderr)
        return 2
    if args.calibrate_copy:
        a = torch.full((1 << 30,), 1, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": 1 << 30, "copies": 3}))
        return 0
    from paper_2306_16384_amd.build import ensure_built
    ensure_built()
    gids.lib()
    if args.probe_box:
        print(json.dumps(probe_box(torch, gids)))
        return 0
    wl.native.build()

    shared = dict(torch=torch, wl=wl, gids=gids, GatherSession=GatherSession)
    result = run_workload(args, shared)
    if result is None:                                          # a sweep printed its own object
        if "world" in shared:
            gids.gids_store_destroy(shared.pop("world")["store"])
        return 0
    # auto: only for the bare command (no option besides --gpus / --steps / --warmup), i.e. the default benchmark line
    given = {a.split("=")[0] for a in sys.argv[1:] if a.startswith("--")}
    plain = given <= {"--gpus", "--steps", "--warmup"}
    if args.others == "on" or (args.others == "auto" and plain):
        # the other configurations in the same line: the HBM-bound one, the mid-size one and the launch-bound one
        import copy
        result["other_workloads"] = {}
        # (tiny and medium twice: call by call, and 32 iterations merged per call, Section 3.2's remedy for
        # minibatches that are small beside the cost of launching and ordering their kernels)
        # (and Large and Medium once more in merged calls in which a CPU-buffer row that several steps of a call need
        # crosses the link once: gids_cache_set_group_dedup, outside the per-minibatch cost model)
        for name in ("large_merged", "large_merged_dedup", "skew", "skew_merged", "resident", "medium", "medium_merged",
                     "medium_merged_dedup", "tiny", "tiny_merged"):
            if name == args.workload:
                continue
            sub = copy.copy(args)
            sub.workload, sub.steps, sub.warmup, sub.cpu_seconds = name, min(args.steps, 20), min(args.warmup, 6), 4.0
            if name == "tiny_merged":
                sub.workload, sub.accum, sub.many, sub.steps, sub.warmup = "tiny", 1, 32, 1280, 32
            elif name == "medium_merged":
                sub.workload, sub.accum, sub.many, sub.steps, sub.warmup = "medium", 1, 32, 320, 32
            elif name in ("large_merged", "large_merged_dedup"):
                sub.workload, sub.accum, sub.many, sub.steps, sub.warmup = "large", 1, 16, 96, 32
                sub.group_dedup = name.endswith("dedup")
                if sub.group_dedup:                             # (the more steps per call, the more rows they share)
                    sub.many, sub.steps = 32, 128
                sub.cpu_seconds = 14.0                          # (the oracle replays the warm-up before it can compare)
            elif name == "medium_merged_dedup":
                sub.workload, sub.accum, sub.many, sub.group_dedup, sub.steps, sub.warmup = "medium", 1, 32, True, 320, 32
            elif name == "skew_merged":
                sub.workload, sub.accum, sub.many, sub.steps, sub.warmup = "skew", 1, 32, 192, 32
            elif name in ("skew", "medium"):
                sub.steps, sub.warmup = 60, 16
            elif name == "tiny":
                sub.steps, sub.warmup = 320, 32
            log(f"--- other workload: {name}")
            r = run_workload(sub, shared)
            result["other_workloads"][name] = {
                "merged_calls_of": sub.many, "group_dedup": bool(sub.group_dedup),
                "weighted_roofline_frac_of_bytes_moved": r["weighted_roofline"]["frac_of_bytes_moved"],
                "value": r["value"], "unit": r["unit"], "ms_per_step": r["ms_per_step"], "steps": r["steps"],
                "unique_ids_per_s": r["unique_ids_per_s"], "workload": r["config"]["workload"],
                "per_step": r["per_step"], "weighted_roofline_frac": r["weighted_roofline"]["frac"],
                "roofline": {k: r["roofline"][k] for k in ("bound", "achieved", "peak", "unit", "frac", "avg_ms")},
                "oracle_count_mismatches": r.get("cpu_baseline", {}).get("count_mismatches_vs_gpu"),
                "oracle_minibatches_compared": r.get("cpu_baseline", {}).get("minibatches_compared"),
                "check": r.get("check")}
    if "world" in shared:
        gids.gids_store_destroy(shared.pop("world")["store"])
    print(json.dumps(result))
    return 0


def probe_box(torch, gids):
    """The machine's own ceilings, measured through the library's C ABI and plain device copies."""
    import glob
    res = {"host_cores": os.cpu_count(), "omp_num_threads": os.environ.get("OMP_NUM_THREADS")}
    for line in open("/proc/meminfo"):
        if line.startswith("MemTotal"):
            res["host_memory_GiB"] = int(line.split()[1]) / 2**20
    link = {}
    for f in glob.glob("/sys/class/drm/card*/device/current_link_speed") + glob.glob("/sys/class/drm/card*/device/current_link_width"):
        try:
            link[f.split("/")[4] + "/" + os.path.basename(f)] = open(f).read().strip()
        except OSError:
            pass
    res["pcie_link"] = link
    props = torch.cuda.get_device_properties(0)
    res["device"] = {"name": props.name, "compute_units": props.multi_processor_count, "memory_GiB": props.total_memory / 2**30}
    # pinned host memory: stores of 8 GiB until the runtime refuses, then one store of everything that was granted
    chunk_rows, R, stores = (8 << 30) // 2048, 2048, []
    try:
        while len(stores) < 40:
            try:
                stores.append(gids.gids_store_create(chunk_rows, R, 8))
            except gids.GidsError as e:
                res["pinned_chunks_refused_after_GiB"] = 8 * len(stores)
                res["pinned_refusal"] = str(e)
                break
        else:
            res["pinned_chunks_refused_after_GiB"] = None
    finally:
        for st in stores:
            gids.gids_store_destroy(st)
    granted = res.get("pinned_chunks_refused_after_GiB") or 320
    for gib in (granted + 8, granted):
        try:
            st = gids.gids_store_create((gib << 30) // R, R, 8)
            gids.gids_store_destroy(st)
            res[f"single_store_of_{gib}_GiB"] = "granted"
        except gids.GidsError as e:
            res[f"single_store_of_{gib}_GiB"] = "refused"
    # the link as the row mover's launch shape sees it (hashed 2 KiB rows of a 16 GiB table, zero-copy)
    st = gids.gids_store_create((16 << 30) // R, R, 8)
    try:
        rate, overhead = gids.gids_store_calibrate(st)
        res["zero_copy_hashed_2KiB_rows_GBs"] = rate * R / 1e9
        res["zero_copy_overhead_us"] = overhead * 1e6
    finally:
        gids.gids_store_destroy(st)

    def timed(fn, nbytes, reps=5):
        fn()
        torch.cuda.synchronize()
        best = 1e9
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) * 1e-3)
        return nbytes / best / 1e9

    host = torch.empty(1 << 30, dtype=torch.uint8).pin_memory()
    dev = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    res["copy_host_to_device_1GiB_GBs"] = timed(lambda: dev.copy_(host, non_blocking=True), 1 << 30)
    res["copy_device_to_host_1GiB_GBs"] = timed(lambda: host.copy_(dev, non_blocking=True), 1 << 30)
    a = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
    b = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
    res["copy_device_to_device_2GiB_read_plus_write_GBs"] = timed(lambda: b.copy_(a), 2 * (2 << 30))
    res["fill_device_2GiB_write_GBs"] = timed(lambda: b.fill_(1), 2 << 30)
    res["sum_device_2GiB_read_GBs"] = timed(lambda: a.view(torch.int64).sum(), 2 << 30)
    return res


def run_workload(args, shared):
    """Sets one configuration up (table pinned and filled, graph, hot nodes, ID lists), runs it, releases the
    table; returns the result object (None after a sweep, which prints its own)."""
    torch, wl, gids, GatherSession = shared["torch"], shared["wl"], shared["gids"], shared["GatherSession"]
    base = wl.CONFIGS[args.workload]
    def with_dim(c):
        if not args.dim:
            return c
        from dataclasses import replace
        new_r = args.dim * np.dtype(c.feat_dtype).itemsize
        return replace(c, dim=args.dim, line_bytes=new_r,
                       cache_lines=max(c.ways, c.cache_lines * c.line_bytes // new_r // c.ways * c.ways))

    cfg = with_dim(wl.scaled(base, args.nodes) if args.nodes else pick_scale(base, wl, args.max_pinned_gib))

    def world_key(c):
        """what the pinned table, the graph and the hot nodes depend on: configurations that agree in it share them"""
        return (c.seed, c.n_nodes, c.row_bytes, c.index_dtype, c.dim, c.feat_dtype, c.ell, c.p4, c.d_max, c.cpu_rows,
                args.hot_by, (tuple(c.fanouts), c.n_seeds) if args.hot_by != "indegree" else None)

    world = shared.get("world")
    if world is not None and world["key"] != world_key(cfg):    # (a box pins 64 GiB: one table at a time)
        torch.cuda.synchronize()
        gids.gids_store_destroy(world["store"])
        world = None
        shared.pop("world")
    # pin the store first: a box that grants less pinned memory than assumed runs at half the node count, and so on
    while world is None:
        try:
            store = gids.gids_store_create(cfg.n_nodes, cfg.row_bytes, np.dtype(cfg.index_dtype).itemsize)
            break
        except gids.GidsError as e:
            if e.code != gids.GIDS_E_NOMEM or cfg.n_nodes < 100_000:
                raise
            log(f"cannot pin {cfg.n_nodes * cfg.row_bytes / 1e9:.1f} GB of host memory; halving the node count")
            cfg = with_dim(wl.scaled(base, cfg.n_nodes // 2))
    if args.cache_lines:
        from dataclasses import replace
        cfg = replace(cfg, cache_lines=max(cfg.ways, args.cache_lines // cfg.ways * cfg.ways))
    if args.rows_per_line > 1:
        from dataclasses import replace
        P = args.rows_per_line
        cfg = replace(cfg, line_bytes=P * cfg.row_bytes,
                      cache_lines=max(cfg.ways, cfg.cache_lines * cfg.line_bytes // (P * cfg.row_bytes) // cfg.ways * cfg.ways))
    R = cfg.row_bytes
    if world is not None:
        log(f"workload {cfg.name}: table, graph and hot nodes of the run before")
        store, g, hot, table, rate, overhead = (world[k] for k in ("store", "g", "hot", "table", "rate", "overhead"))
        env = dict(shared, link_rows_per_s=rate, link_overhead_s=overhead, g=g, hot=hot, table=table, store=store, base=base)
        try:
            return run_lists(args, env, cfg, base, g, wl, gids)
        finally:
            if "push_stream" in env:
                shared["push_stream"] = env["push_stream"]
            torch.cuda.synchronize()
    rate, overhead = gids.gids_store_calibrate(store)
    log(f"link calibration: {rate * R / 1e9:.1f} GB/s ({rate / 1e6:.1f} M rows/s), overhead {overhead * 1e6:.1f} us; "
        f"Eq. 2-3: {gids.gids_accum_threshold(rate, overhead, 0.0, 0.95):.0f} link rows in flight for 95 % of it")
    log(f"workload {cfg.name}: N={cfg.n_nodes} R={R} lines={cfg.cache_lines} ways={cfg.ways} L={cfg.line_bytes} "
        f"cpu_rows={cfg.cpu_rows} fanouts={cfg.fanouts} seeds={cfg.n_seeds}")
    t0 = time.time()
    g = wl.make_graph(cfg.seed, cfg.n_nodes, cfg.ell, cfg.p4, cfg.d_max, np.dtype(cfg.index_dtype), native=True)
    log(f"graph: {g.n_edges} edges, mean degree {g.n_edges / g.n:.2f} ({time.time() - t0:.1f} s)")
    t0 = time.time()
    if args.hot_by != "indegree" and cfg.cpu_rows:
        from paper_2306_16384_amd.session import GraphSampler
        with GraphSampler(g.indptr, g.indices) as gs_rank:
            t1 = time.time()
            if args.hot_by == "visits":
                scores = gs_rank.visit_scores(cfg.fanouts, cfg.n_seeds)
            else:
                scores = gs_rank.reverse_pagerank(55705, 20)         # damping 0.85, 20 power iterations
            scores = scores.cpu().numpy().view(np.uint64)
            log(f"{args.hot_by} scores on the GPU: {time.time() - t1:.2f} s")
        hot = wl.top_k_by_score(scores, cfg.cpu_rows)
        del scores
    else:
        hot = wl.hot_nodes(g, cfg.cpu_rows)
    log(f"hot nodes by {args.hot_by}: {len(hot)} ({time.time() - t0:.1f} s)")
    table = wl.normal_table(np.dtype(cfg.feat_dtype))
    t0 = time.time()
    wl.fill_store(cfg.seed, cfg.n_nodes, cfg.dim, table, gids.gids_store_host_ptr(store))
    log(f"store: {cfg.n_nodes * R / 1e9:.2f} GB pinned and filled ({time.time() - t0:.1f} s)")
    env = dict(shared, link_rows_per_s=rate, link_overhead_s=overhead, g=g, hot=hot, table=table, store=store, base=base)
    shared["world"] = dict(key=world_key(cfg), store=store, g=g, hot=hot, table=table, rate=rate, overhead=overhead)
    try:
        return run_lists(args, env, cfg, base, g, wl, gids)
    finally:
        if "push_stream" in env:
            shared["push_stream"] = env["push_stream"]          # one push stream for the whole process
        torch.cuda.synchronize()


def run_lists(args, env, cfg, base, g, wl, gids):

    if args.sweep_skew:
        # the skew sweep: seed IDs Zipf(s) over a seeded permutation of the nodes, window depth 0 / 4 / 16
        points = []
        for s_exp in (0.0, 0.8, 1.2):
            rank_table = wl.synth.zipf_rank_table(cfg.n_nodes, s_exp)
            n_b = args.warmup + 2 * args.steps + 16 + 1
            t0 = time.time()
            raws = [wl.sample_minibatch(g, cfg.seed, b, cfg.fanouts, cfg.n_seeds, rank_table) for b in range(n_b)]
            log(f"zipf s={s_exp}: sampled {n_b} minibatches ({time.time() - t0:.1f} s)")
            # every point twice: the configuration's cache (which nothing leaves within a few hundred minibatches,
            # so the window has nothing to protect) and one of 2,048 sets, a few minibatches' misses large, where
            # lines are evicted inside the run and the hit ratio moves with the depth
            from dataclasses import replace
            small = replace(cfg, cache_lines=2048 * cfg.ways)
            for label, c in (("configuration", cfg), ("under eviction pressure", small)):
                for w in (0, 4, 16):
                    res = run_point(args, env, c, w, raws, 0)
                    per = res["per_step"]
                    points.append({"zipf_s": s_exp, "window": w, "cache": label, "cache_lines": c.cache_lines,
                                   "gathered_GBs": res["value"], "hit_rate": per["hit"] / max(1.0, per["unique"]),
                                   "hit_rate_of_cache_traffic": per["hit"] / max(1.0, per["unique"] - per["cpu_hit"]),
                                   "cpu_buffer_rate": per["cpu_hit"] / max(1.0, per["unique"]),
                                   "ms_per_step": res["ms_per_step"],
                                   "weighted_roofline_frac": res["weighted_roofline"]["frac"],
                                   "oracle_count_mismatches": res.get("cpu_baseline", {}).get("count_mismatches_vs_gpu")})
                    log(json.dumps(points[-1]))
        print(json.dumps({"metric": "skew sweep: gathered GB/s and hit rate per (zipf s, window depth)", "n_gpus": 1,
                          "config": {"workload": cfg.name, "n_nodes": cfg.n_nodes, "steps": args.steps,
                                     "warmup": args.warmup}, "points": points}))
        return None

    window = cfg.window if args.window < 0 else args.window
    prewarm = args.prewarm if args.prewarm >= 0 else (1_000_000 if args.workload == "resident" else 0)
    n_pre = (cfg.n_nodes + prewarm - 1) // prewarm if prewarm else 0
    passes = 3 if args.consumer_ms > 0 else 2                           # timed, event-timed (, with a consumer)
    n_batches = n_pre + args.warmup + passes * args.steps + window + 1  # + look-ahead
    rank_table = wl.synth.zipf_rank_table(cfg.n_nodes, cfg.seed_zipf_s) if cfg.seed_zipf_s is not None else None
    t0 = time.time()
    raws = [np.arange(b * prewarm, min(cfg.n_nodes, (b + 1) * prewarm), dtype=np.int64) for b in range(n_pre)]
    if args.layerwise:
        layer_sizes = tuple(int(x) for x in args.layerwise.split(","))
        for b in range(n_batches - n_pre):
            raws.append(wl.layerwise_minibatch(g, cfg.seed, b, layer_sizes, cfg.n_seeds))
            if b % 8 == 7:
                log(f"layer-wise lists: {b + 1} of {n_batches - n_pre} ({time.time() - t0:.0f} s)")
    else:
        raws += [wl.sample_minibatch(g, cfg.seed, b, cfg.fanouts, cfg.n_seeds, rank_table) for b in range(n_batches - n_pre)]
    log(f"sampled {n_batches - n_pre} minibatches, raw IDs per minibatch <= {max(len(r) for r in raws)} "
        f"({time.time() - t0:.1f} s)")
    for k in range(args.repeat - 1):
        res = run_point(args, env, cfg, window, raws, n_pre)
        log(f"repeat {k + 1} of {args.repeat}: {res['ms_per_step']:.4f} ms per step, "
            f"weighted roofline {res['weighted_roofline']['frac']:.4f}, phases {res['roofline']['phase_ms']}")
    return run_point(args, env, cfg, window, raws, n_pre)


def run_point(args, env, cfg, window, raws, n_pre):
    """One timed run of `cfg` with window depth `window` over the raw ID lists `raws`
    (the first n_pre of them pre-warm lists)."""
    torch, wl, gids, GatherSession = env["torch"], env["wl"], env["gids"], env["GatherSession"]
    hot, table, base = env["hot"], env["table"], env["base"]
    R = cfg.row_bytes
    steps, warmup = args.steps, args.warmup + n_pre
    n_batches = warmup + (3 if args.consumer_ms > 0 else 2) * steps + window + 1
    assert len(raws) >= n_batches
    max_raw = max(len(r) for r in raws[:n_batches])
    t0 = time.time()
    ses = GatherSession(cfg.n_nodes, R, np.dtype(cfg.index_dtype), cfg.cache_lines, cfg.ways, cfg.line_bytes, window,
                        args.accum, store_handle=env["store"])
    ses.pin_hot(hot)
    ses.reserve(max_raw)
    if args.policy == "random":
        ses.set_policy(gids.GIDS_POLICY_RANDOM, cfg.seed)
    if args.rows_per_line > 1:
        ses.set_rows_per_line(args.rows_per_line)
    if args.accum and args.accum_adaptive:
        ses.set_accum_mode(gids.GIDS_ACCUM_ADAPTIVE)
    if args.group_dedup:
        ses.set_group_dedup(True)
    log(f"cache W={window}: created, CPU buffer {len(hot) * R / 1e9:.2f} GB pinned ({time.time() - t0:.1f} s)")
    dev = [ses.to_device(r) for r in raws[:n_batches]]
    sampler = None
    if args.gpu_sampler and args.layerwise:
        raise SystemExit("--gpu-sampler draws neighbourhood samples; it cannot be combined with --layerwise")
    if args.gpu_sampler:
        from paper_2306_16384_amd.session import GraphSampler
        g = env["g"]
        t0 = time.time()
        sampler = GraphSampler(g.indptr, g.indices, zero_copy=args.sampler_zero_copy)
        cap_raw = sampler.capacity(cfg.fanouts, cfg.n_seeds)
        ses.reserve(max(max_raw, cap_raw))
        n_slots = window + 3
        raw_bufs = [torch.empty(cap_raw, dtype=ses.torch_id, device="cuda") for _ in range(n_slots)]
        n_bufs = [torch.zeros(1, dtype=torch.int32, device="cuda") for _ in range(n_slots)]
        log(f"GPU sampler: graph {'pinned for zero-copy' if args.sampler_zero_copy else 'copied to HBM'} ({(g.indptr.nbytes + g.indices.nbytes) / 1e9:.2f} GB, "
            f"{time.time() - t0:.1f} s), raw capacity {cap_raw} IDs per minibatch")
    cap_rows = max(len(np.unique(r)) for r in raws[:n_batches])
    # outputs rotate; with the accumulator on, an output must survive until the flush that completes it
    # (a group holds at most GIDS_ACCUM_MAX_MERGE = 32 minibatches, so a buffer is complete before its turn comes again)
    ring = 2 if args.accum == 0 else 40
    outs = [torch.empty((cap_rows, R), dtype=torch.uint8, device="cuda") for _ in range(ring)]
    uniqs = [torch.empty(cap_rows, dtype=ses.torch_id, device="cuda") for _ in range(ring)]
    torch.cuda.synchronize()

    # pushes go to their own stream (where a sampler would produce ID lists), gathers to the consumer's:
    # the library then overlaps the classification of minibatch t + 1 with the row movement of minibatch t
    # small caches: the library does not overlap (unless GIDS_PIPELINE=1 forces its internal stream on)
    small = cfg.cache_lines * cfg.line_bytes < (32 << 20) and os.environ.get("GIDS_PIPELINE", "0") == "0"
    # (merged calls classify on the library's internal stream whatever the cache size: their pushed lists come on a
    # stream of their own as well, or the next call's classification would wait for this call's rows)
    one_stream = args.one_stream or (small and not args.many)
    # One push stream for the whole process: HIP multiplexes streams onto a few hardware queues in creation
    # order, and a push stream that lands on the gather stream's queue has its event markers stuck behind the
    # row mover, which serialises the two (seen with the sixth stream created in a sweep).
    if "push_stream" not in env:
        env["push_stream"] = torch.cuda.Stream()
    push_stream = torch.cuda.current_stream() if one_stream else env["push_stream"]
    pushed = 0

    # At depth 0 the list of minibatch t is still pushed just before its gather (it pins nothing), so that its
    # deduplication overlaps the previous row movement like every other depth's; --pass-ids at depth 0 is the
    # plain call without any push.
    use_push = window > 0 or not args.pass_ids

    def keep_window_full(t):
        nonlocal pushed
        while use_push and pushed < n_batches and pushed <= t + window:
            if sampler is not None and pushed >= n_pre:         # list number pushed - n_pre of the sampled sequence
                k = pushed % n_slots
                sampler.sample(cfg.seed, pushed - n_pre, cfg.fanouts, cfg.n_seeds, raw_bufs[k], n_bufs[k],
                               stream=push_stream)
                ses.push_dev(raw_bufs[k], n_bufs[k], stream=push_stream)
            else:
                ses.push(dev[pushed], stream=push_stream)
            pushed += 1

    def step(t):
        keep_window_full(t)                                     # push of minibatch t + W (+1 at start-up)
        return ses.gather(dev[t] if args.pass_ids else None, outs[t % ring], uniqs[t % ring])

    def steps_merged(t0, t1, seqs_out):
        """minibatches [t0, t1) through gids_gather_many, args.many at a time"""
        nonlocal pushed
        t = t0
        while t < t1:
            k = min(args.many, t1 - t)
            pushes = []
            for i in range(k):
                if pushed < n_batches and pushed <= t + i + window:
                    pushes.append(dev[pushed])
                    pushed += 1
                else:
                    pushes.append(None)
            seq0 = ses.gather_many(pushes, [outs[(t + i) % ring] for i in range(k)],
                                   [uniqs[(t + i) % ring] for i in range(k)], push_stream=push_stream)
            for i in range(k):
                seqs_out[t + i] = seq0 + i
            t += k

    if args.many:
        if not args.accum or sampler is not None or args.pass_ids or not use_push:
            raise SystemExit("--many needs --accum > 0 and the plain push / gather loop")

    seqs = {}
    if args.many:
        while pushed < min(n_batches, window):                  # the look-ahead, before the first merged call
            ses.push(dev[pushed], stream=push_stream)
            pushed += 1
        torch.cuda.current_stream().wait_stream(push_stream)
        steps_merged(0, warmup, seqs)
    else:
        for t in range(warmup):
            seqs[t] = step(t)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    if args.many:
        steps_merged(warmup, warmup + steps, seqs)
    else:
        for t in range(warmup, warmup + steps):
            seqs[t] = step(t)
    ses.flush()
    torch.cuda.current_stream().wait_stream(push_stream)       # the timed region ends when its pushes have too
    e1.record()
    torch.cuda.synchronize()
    total_ms = e0.elapsed_time(e1)

    stats = {t: ses.stats(seqs[t]) for t in range(max(0, warmup + steps - 60), warmup + steps)}
    timed = [stats[t] for t in range(warmup, warmup + steps) if t in stats]
    if len(timed) != steps:
        log("note: only the last 60 gathers keep their counters; use --steps <= 60 for exact accounting")
    n_unique = sum(s.n_unique for s in timed)
    n_hit = sum(s.n_hit for s in timed)
    n_cpu = sum(s.n_cpu_hit for s in timed)
    n_miss = sum(s.n_miss for s in timed)
    n_byp = sum(s.n_bypass for s in timed)
    n_again = sum(s.n_cpu_again for s in timed)                 # CPU-buffer rows that came as a copy inside device memory
    scale = steps / max(1, len(timed))
    # Bytes the method must move.  One row per line: a miss's row is read once and written to the output and
    # to its line.  Several rows per line: a filled line is read from the store and written to the cache in
    # full, and contains every missed row of that line, so only CPU-buffer rows and bypassed rows cross the
    # link besides; every missed row is still written to the output.
    P = args.rows_per_line
    n_fills = sum(s.n_line_fills for s in timed)

    def algorithmic_bytes(hit, cpu, miss, byp, fills):
        if P == 1:
            return (cpu + miss) * R, (2 * hit + cpu + 2 * (miss - byp) + byp) * R
        return (cpu + byp + fills * P) * R, (2 * hit + cpu + miss + fills * P) * R

    link_bytes, hbm_bytes = (x * scale for x in algorithmic_bytes(n_hit, n_cpu, n_miss, n_byp, n_fills))
    gathered_bytes = n_unique * R * scale
    t_roof_ms = (link_bytes / (LINK_PEAK_GBS * 1e9) + hbm_bytes / (HBM_PEAK_GBS * 1e9)) * 1e3
    t_overlap_ms = max(link_bytes / (LINK_PEAK_GBS * 1e9), hbm_bytes / (HBM_PEAK_GBS * 1e9)) * 1e3
    value = gathered_bytes / (total_ms * 1e-3) / 1e9

    # second pass with per-phase HIP events (on the launch stream) for the row mover's own roofline
    gids.gids_profile_enable(ses.cache, True)
    pseq = {}
    if args.many:
        steps_merged(warmup + steps, warmup + 2 * steps, pseq)
    else:
        for t in range(warmup + steps, warmup + 2 * steps):
            pseq[t] = step(t)
    ses.flush()
    torch.cuda.synchronize()
    gids.gids_profile_enable(ses.cache, False)
    keep = sorted(pseq)[-min(steps, 60):]
    if args.many:                                               # merged calls record no per-gather phase events:
        ph = np.zeros((len(keep), 3))                           # the step time of this pass stands in for the mover's
        ph[:, 2] = total_ms / steps
    else:
        ph = np.array([gids.gids_profile_read(ses.cache, pseq[t]) for t in keep])
    pst = [ses.stats(pseq[t]) for t in keep]
    mv_ms = float(ph[:, 2].mean())
    per_launch = [algorithmic_bytes(s.n_hit, s.n_cpu_hit, s.n_miss, s.n_bypass, s.n_line_fills) for s in pst]
    mv_link = np.mean([b[0] for b in per_launch])
    mv_hbm = np.mean([b[1] for b in per_launch])
    link_bound = mv_link / LINK_PEAK_GBS >= mv_hbm / HBM_PEAK_GBS
    if link_bound:
        roof = {"bound": "host_link", "achieved": mv_link / (mv_ms * 1e-3) / 1e9, "peak": LINK_PEAK_GBS}
    else:
        roof = {"bound": "hbm", "achieved": mv_hbm / (mv_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS}
    roof.update({"unit": "GB/s", "frac": roof["achieved"] / roof["peak"], "traffic": None, "traffic_reference": TRAFFIC_REFERENCE.get(base.name),
                 "kernel": "move_kernel", "avg_ms": mv_ms, "link_bytes_per_launch": float(mv_link),
                 "hbm_bytes_per_launch": float(mv_hbm),
                 "phase_ms": {"dedup": float(ph[:, 0].mean()), "probe_victim": float(ph[:, 1].mean()), "move": mv_ms}})

    overlap = None
    if args.consumer_ms > 0:
        # A stand-in for the training step: matmuls that keep every CU busy, ordered after the gather they
        # consume; the gather of the next minibatch is free to run beside them.
        if "consumer_stream" not in env:
            env["consumer_stream"] = torch.cuda.Stream()
        cs = env["consumer_stream"]
        ma = torch.randn(4096, 4096, device="cuda", dtype=torch.bfloat16)
        mb = torch.randn(4096, 4096, device="cuda", dtype=torch.bfloat16)
        mc = torch.empty(4096, 4096, device="cuda", dtype=torch.bfloat16)
        sink = torch.zeros(1, device="cuda", dtype=torch.float32)

        def consume(rows, reps):
            sink.add_(rows[:256].float().sum())                 # touches the gathered rows
            for _ in range(reps):
                torch.mm(ma, mb, out=mc)

        def timed(fn):
            torch.cuda.synchronize()
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a0.record()
            fn()
            torch.cuda.current_stream().wait_stream(cs)
            torch.cuda.current_stream().wait_stream(push_stream)
            a1.record()
            torch.cuda.synchronize()
            return a0.elapsed_time(a1)

        def only_consumer(reps):
            def run():
                cs.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(cs):
                    for k in range(steps):
                        consume(outs[k % ring], reps)
            return run

        timed(only_consumer(4))                                 # warm-up (library handles, clocks)
        per_mm = timed(only_consumer(4)) / (steps * 4)
        reps = max(1, int(round(args.consumer_ms / per_mm)))
        cons_ms = timed(only_consumer(reps)) / steps
        produced = [torch.cuda.Event() for _ in range(ring)]
        consumed = [torch.cuda.Event() for _ in range(ring)]
        first = warmup + 2 * steps

        def both():
            for t in range(first, first + steps):
                k = t % ring
                if t >= first + ring:
                    torch.cuda.current_stream().wait_event(consumed[k])   # the buffer is free again
                pseq[t] = step(t)
                produced[k].record()
                cs.wait_event(produced[k])
                with torch.cuda.stream(cs):
                    consume(outs[k], reps)
                    consumed[k].record()
            ses.flush()

        gids.gids_profile_enable(ses.cache, True)
        both_ms = timed(both) / steps
        gids.gids_profile_enable(ses.cache, False)
        ph_both = np.array([gids.gids_profile_read(ses.cache, pseq[t]) for t in sorted(pseq)[-min(steps, 60):]])
        gather_ms = total_ms / steps
        overlap = {"consumer": f"{reps} bf16 4096^3 matmuls per minibatch on a stream of its own, after a read of the gathered rows",
                   "consumer_alone_ms": cons_ms, "gather_alone_ms": gather_ms, "both_ms_per_step": both_ms,
                   "serial_sum_ms": cons_ms + gather_ms, "ideal_overlap_ms": max(cons_ms, gather_ms),
                   "hidden_fraction_of_the_shorter": (cons_ms + gather_ms - both_ms) / min(cons_ms, gather_ms),
                   "move_kernel_ms_beside_consumer": float(ph_both[:, 2].mean()), "move_kernel_ms_alone": mv_ms,
                   "classify_ms_beside_consumer": float(ph_both[:, 1].mean()), "classify_ms_alone": float(ph[:, 1].mean())}
        log(f"overlap with a consumer: {json.dumps(overlap)}")

    result = {
        "metric": "gathered feature GB/s per minibatch (distinct IDs x row bytes / time), steady state",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": total_ms / steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "unique_ids_per_s": n_unique * scale / (total_ms * 1e-3),
        "config": {"workload": cfg.name, "n_nodes": cfg.n_nodes, "row_bytes": R, "cache_lines": cfg.cache_lines,
                   "ways": cfg.ways, "line_bytes": cfg.line_bytes, "cpu_buffer_rows": cfg.cpu_rows, "window": window,
                   "fanouts": list(cfg.fanouts), "seeds_per_batch": cfg.n_seeds, "accum_threshold": args.accum, "accum_adaptive": bool(args.accum_adaptive), "merged_calls_of": args.many, "group_dedup": bool(args.group_dedup), "merged_calls_through": dict(zip(("merged_kernels", "per_step_kernels"), gids.gids_cache_many_calls(ses.cache))) if args.many else None, "prewarm_lists": n_pre, "gpu_sampler": bool(args.gpu_sampler), "policy": args.policy, "hot_by": args.hot_by, "rows_per_line": args.rows_per_line, "id_stream": ("layerwise " + args.layerwise) if args.layerwise else "neighbourhood",
                   "id_dtype": cfg.index_dtype, "scaled_from": base.n_nodes if cfg.n_nodes != base.n_nodes else None},
        "per_step": {"unique": n_unique * scale / steps, "hit": n_hit * scale / steps, "cpu_hit": n_cpu * scale / steps,
                     "miss": n_miss * scale / steps, "bypass": n_byp * scale / steps,
                     "line_fills": n_fills * scale / steps, "cpu_again": n_again * scale / steps},
        "weighted_roofline": {"hbm_peak_GBs": HBM_PEAK_GBS, "link_peak_GBs": LINK_PEAK_GBS,
                              "t_roof_ms_per_step": t_roof_ms / steps, "frac": t_roof_ms / total_ms,
                              "frac_overlap_bound": t_overlap_ms / total_ms,
                              "roofline_gathered_GBs": gathered_bytes / (t_roof_ms * 1e-3) / 1e9,
                              # the same with the bytes that really moved: a CPU-buffer row that came as a copy
                              # (gids_cache_set_group_dedup) is R less over the link and R more out of HBM
                              "frac_of_bytes_moved": ((link_bytes - n_again * scale * R) / (LINK_PEAK_GBS * 1e9) +
                                                      (hbm_bytes + n_again * scale * R) / (HBM_PEAK_GBS * 1e9)) * 1e3 / total_ms},
        "roofline": roof,
        "link_calibration": {"GBs": env["link_rows_per_s"] * R / 1e9, "overhead_us": env["link_overhead_s"] * 1e6,
                             "rows_for_95pct_eq2_3": gids.gids_accum_threshold(env["link_rows_per_s"],
                                                                                env["link_overhead_s"], 0.0, 0.95),
                             "link_rows_per_step": (n_cpu + n_miss) * scale / steps},
    }
    if overlap is not None:
        result["overlap_with_consumer"] = overlap

    if sampler is not None:
        # the sampler alone: back-to-back minibatches on one stream, and the oracle's sampler on the host
        n_s = min(20, n_batches - n_pre)
        torch.cuda.synchronize()
        s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s0.record()
        for b in range(n_s):
            sampler.sample(cfg.seed, b, cfg.fanouts, cfg.n_seeds, raw_bufs[0], n_bufs[0])
        s1.record()
        torch.cuda.synchronize()
        gpu_ms = s0.elapsed_time(s1) / n_s
        last = raw_bufs[0][:int(n_bufs[0].item())].cpu().numpy().astype(np.int64)
        raw_ids = float(np.mean([len(r) for r in raws[n_pre:n_pre + n_s]]))
        result["sampler"] = {"gpu_ms_per_minibatch": gpu_ms, "raw_ids_per_minibatch": raw_ids,
                             "raw_ids_per_s": raw_ids / (gpu_ms * 1e-3),
                             "graph": "CSR in pinned host memory, zero-copy" if args.sampler_zero_copy else "CSR in HBM",
                             "list_equals_reference": bool(np.array_equal(last, raws[n_pre + n_s - 1]))}
        if not args.no_cpu:
            import oracle
            og = oracle.Graph(cfg.seed, cfg.n_nodes, csr=(env["g"].indptr, env["g"].indices))
            t0 = time.perf_counter()
            n_o = 0
            while n_o < n_s and time.perf_counter() - t0 < 10.0:
                og.sample(cfg.seed, n_o, cfg.fanouts, cfg.n_seeds)
                n_o += 1
            result["sampler"]["cpu_oracle_ms_per_minibatch"] = (time.perf_counter() - t0) / n_o * 1e3
            del og

    # sampled check of the timed configuration against the definition (row = closed-form feature row)
    if not args.no_check:
        import oracle
        t_last = max(pseq)                                        # the last minibatch gathered
        st = ses.stats(pseq[t_last])
        u = uniqs[t_last % ring][:st.n_unique].cpu().numpy().astype(np.int64)
        assert np.array_equal(u, np.unique(raws[t_last])), "distinct-ID list differs from sort-unique of the input"
        pick = np.unique(np.linspace(0, len(u) - 1, 64).astype(np.int64))
        got = outs[t_last % ring][torch.from_numpy(pick).cuda()].cpu().numpy()
        want = oracle.feat_rows(cfg.seed, u[pick], cfg.dim, table).view(np.uint8).reshape(len(pick), R)
        assert np.array_equal(got, want), "gathered rows differ from the closed-form feature rows"
        result["check"] = f"last minibatch: ID list exact, {len(pick)} sampled rows equal the oracle's closed form"

    # the oracle on this machine's host cores, same ID lists, bounded time
    if not args.no_cpu:
        import oracle
        oracle.build()
        store_np = ses.store_view()
        # (a simulated cache beyond 16 GiB of host memory is left out: the oracle then runs without its data
        # plane, counters only, and its rate excludes the row copies)
        with_rows = cfg.cache_lines * cfg.line_bytes <= (16 << 30)
        sim = oracle.Sim(cfg.n_nodes, cfg.cache_lines, cfg.ways, window, R, cfg.line_bytes,
                         store_np if with_rows else None)
        sim.set_hot(hot)
        if args.rows_per_line > 1:
            sim.set_rows_per_line(args.rows_per_line)
        if args.policy == "random":
            sim.set_policy(1, cfg.seed)
        if args.accum and not args.many:
            sim.set_accum(args.accum, 1 if args.accum_adaptive else 0)
        opushed, done, o_unique, o_time = 0, 0, 0, 0.0
        mismatches, compared = 0, 0
        budget_end = time.time() + args.cpu_seconds
        for t in range(warmup + steps):
            while window and opushed < n_batches and opushed <= t + window:
                sim.push(raws[opushed])
                opushed += 1
            ts = time.perf_counter()
            u, rows, ost = sim.gather(raws[t])
            dt = time.perf_counter() - ts
            if t in stats:
                compared += 1
                same = tuple(int(x) for x in ost) == stats[t].as_tuple()
                if args.accum and not args.many:                # the accumulator's groups as well
                    same = same and sim.accum_last[:2] == (stats[t].n_pending, stats[t].flushed)
                mismatches += not same
            if t >= min(warmup, 2):                             # skip the cold start like the GPU leg
                o_unique += len(u)
                o_time += dt
                done += 1
            if time.time() > budget_end and done >= 1:
                break
        result["cpu_baseline"] = {
            "value": o_unique * R / o_time / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "unique_ids_per_s": o_unique / o_time, "host_cores_on_box": os.cpu_count(),
            "sample": f"{done} minibatches of this workload (gather only: sort-unique, cache simulation"
                      f"{', row copy' if with_rows else '; no row copies: the simulated cache would not fit'}; "
                      f"window pushes and sampling excluded), single thread",
            "count_mismatches_vs_gpu": mismatches, "minibatches_compared": compared}
        if mismatches:
            log(f"WARNING: {mismatches} minibatches differ from the oracle's counters")
    ses.close()
    if sampler is not None:
        sampler.close()
    return result




if __name__ == "__main__":
    sys.exit(main())
