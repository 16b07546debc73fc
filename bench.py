#!/usr/bin/env python3
"""Benchmark of the RapidGNN data path on one MI355X.

A step is one mini-batch taken through the whole hot path: epoch schedule (once per epoch), k-hop
sampling, access histogram, TopHot + cache fill (once per epoch, amortised over its batches) and the
per-batch feature gather.  `--steps K` with K below one epoch times a K-batch epoch from a cold cache
(schedule, K samples, histogram over them, TopHot, pulls, K gathers); the timed region is repeated
`--reps` times, each from a cold cache, and the median is reported with the spread beside it.  Because
the first batches of an epoch need most of the remote rows, the per-batch time of a short epoch is
dominated by the host link; the rate of the workload's whole epoch is therefore measured in the same run
and reported under "full_epoch", whatever K is.  Kernel durations (roofline) come from one more pass with
the library's hipEvent brackets switched on, outside the timed repetitions.

Inputs are synthetic (seeded Chung-Lu graph, N(0,1) features) and resident in HBM / pinned host memory
before the timed region starts.  Prints one JSON line.
"""
import argparse
import json
import os
import re
import statistics
import sys
import time

# The pipeline keeps up to five streams busy at once (gathers, miss rows, host-link pulls, two more sampler lanes);
# with HIP's default of 4 hardware queues two of them would share a queue and serialise.  A value the user set is kept.
HWQ_SET_BY_USER = "GPU_MAX_HW_QUEUES" in os.environ
if not HWQ_SET_BY_USER:
    os.environ["GPU_MAX_HW_QUEUES"] = "8"

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E peak
HOSTLINK_PEAK_GBS = 64.0   # PCIe Gen5 x16, one direction


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def recorded_traffic(workload):
    """HBM bytes per gathered row from the committed rocprofv3 --pmc summary of this workload's gather kernel, or None.
    The summary file carries one machine-readable line: `bench_traffic_json: {...}`."""
    path = os.path.join(ROOT, "profiles", f"{workload}_gather_hbm_pmc_traffic.txt")
    try:
        text = open(path).read()
    except OSError:
        return None, None
    m = re.search(r"^bench_traffic_json:\s*(\{.*\})\s*$", text, re.M)
    if not m:
        return None, None
    t = json.loads(m.group(1))
    per_row = (t["fetch_kib"] * t["fetch_scale"] + t["write_kib"] * t["write_scale"]) * 1024.0 / t["rows_per_launch"]
    return per_row, os.path.relpath(path, ROOT)


def run_steps(pipe, steps, totals=None, first_epoch=0):
    """Run `steps` batches through the whole path, epoch after epoch (the last epoch may be partial)."""
    import torch

    def account(p, _k):
        if totals is not None:
            nb = p.n_batches
            per = nb // p.period_epochs
            for e in range(p.period_epochs):              # hits and misses of every epoch of the period
                totals["per_epoch"].append(p.stats[e * per:(e + 1) * per].sum(0))
            totals["stats"] += p.stats[:nb].sum(0)
            totals["rows"] += sum(p.sizes[:nb])
            totals["edges"] += p.edge_counts[:nb].sum()
            totals["cached"] += p.cache.num_cached.clone()
            totals["epochs"] += 1
    bpe, E = pipe.batches_per_epoch, pipe.period_epochs
    full, rem = divmod(steps, bpe * E)                    # whole periods, then a shorter one
    if full:
        pipe.run_epochs(first_epoch, full, bpe, on_epoch_done=account)
    if rem:
        pipe.run_epochs(first_epoch + full * E, 1, max(1, rem // E), on_epoch_done=account)
    torch.cuda.current_stream().synchronize()


def new_totals(dev):
    import torch
    return {"stats": torch.zeros(3, dtype=torch.int64, device=dev), "rows": 0,
            "edges": torch.zeros((), dtype=torch.int64, device=dev),
            "cached": torch.zeros(1, dtype=torch.int64, device=dev), "epochs": 0, "per_epoch": []}


def timed_reps(pipe, steps, reps):
    """`reps` repetitions of `steps` batches, each from a cold cache, each bracketed by a device synchronisation."""
    import gc
    import torch
    times = []
    gc.collect()
    gc.freeze()            # the workload's and the pipeline's objects are here to stay: keep full collections off the timed region
    for _ in range(reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(pipe, steps)
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
    return times


def profiled_pass(pipe, steps, dev, only=None):
    """One more repetition with the library's hipEvent brackets on (all kernels, or the listed kernel ids only): per-kernel
    durations and the row statistics."""
    import torch
    from paper_2505_10806_amd import binding as B
    totals = new_totals(dev)
    pipe.profile_select(only)
    pipe.profile_enable(True)
    pipe.profile_reset()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(pipe, steps, totals)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = {name: pipe.profile_read(kid) for name, kid in
            [("gather_hbm", B.RG_K_GATHER_HBM), ("gather_miss", B.RG_K_GATHER_MISS), ("sample", B.RG_K_SAMPLE),
             ("histogram", B.RG_K_HISTOGRAM), ("cache_fill", B.RG_K_CACHE_FILL), ("mean_aggregate", B.RG_K_AGGREGATE)]}
    pipe.profile_enable(False)
    pipe.profile_select(None)
    return dt, prof, totals


def gather_roofline(prof, totals, row_bytes):
    """Algorithmic HBM bytes of the k_gather_hbm launches of a profiled pass over their summed duration."""
    n_local, n_hit, _ = [int(x) for x in totals["stats"].cpu().tolist()]
    g_ms, g_launches = prof["gather_hbm"]
    hbm_rows = n_local + n_hit
    alg_bytes = 2.0 * row_bytes * hbm_rows                       # every HBM-served row is read once and written once
    achieved = alg_bytes / (g_ms * 1e-3) / 1e9 if g_ms > 0 else 0.0
    return {"achieved": achieved, "frac": achieved / HBM_PEAK_GBS, "algorithmic_bytes_per_launch": alg_bytes / max(g_launches, 1),
            "avg_launch_ms": g_ms / max(g_launches, 1), "launches": g_launches, "hbm_rows": hbm_rows}


def spread(times, steps):
    med = statistics.median(times)
    return {"reps": len(times), "median_ms": med * 1e3, "min_ms": min(times) * 1e3, "max_ms": max(times) * 1e3,
            "times_ms": [round(t * 1e3, 3) for t in times],
            "batches_per_s_median": steps / med, "batches_per_s_min": steps / max(times), "batches_per_s_max": steps / min(times)}


def cpu_baseline(wl, n_batches=None, target_s=12.0):
    """The CPU oracle, as it stands, on the first batches of epoch 0 (single thread).  With n_batches None the
    sample is sized for about target_s seconds of CPU work from a two-batch trial run."""
    import numpy as np
    import oracle
    cfg = wl.cfg
    rp = wl.row_ptr.cpu().numpy().astype(np.int64)
    ci = wl.col_idx.cpu().numpy()
    X = wl.features.cpu().numpy()
    home = wl.home.cpu().numpy()
    train = wl.train_ids.cpu().numpy()
    bpe = wl.batches_per_epoch()

    def whole_path(n):
        phases = {"schedule": 0.0, "sample": 0.0, "histogram": 0.0, "tophot_fill": 0.0, "gather": 0.0}
        clock = time.perf_counter
        t0 = t = clock()
        batches = oracle.epoch_batches(train, cfg.batch_size, wl.seed, 0)[:n]
        phases["schedule"] = clock() - t
        counts = np.zeros(cfg.num_nodes, dtype=np.uint32)
        inputs = []
        for seeds in batches:
            t = clock()
            blk = oracle.sample_blocks(rp, ci, seeds, cfg.fanouts, wl.seed, 0)
            phases["sample"] += clock() - t
            t = clock()
            oracle.access_histogram(blk.input_nodes, counts)
            phases["histogram"] += clock() - t
            inputs.append(blk.input_nodes)
        t = clock()
        ids, loc = oracle.build_cache(counts, home, wl.capacity_rows)
        oracle.fill_cache(X, ids, wl.stride)
        phases["tophot_fill"] = clock() - t
        rows = 0
        t = clock()
        for nodes in inputs:
            oracle.gather_features(X, nodes, loc, wl.stride)
            rows += nodes.size
        phases["gather"] = clock() - t
        return len(batches), rows, clock() - t0, phases

    if n_batches is None:
        n, _, dt, _ = whole_path(min(2, bpe))
        n_batches = max(2, min(bpe, int(target_s / max(dt / n, 1e-6))))
    n, rows, dt, phases = whole_path(min(n_batches, bpe))
    return {"value": n / dt, "unit": "batches/s", "cores": 1, "kind": "oracle",
            "sample": f"first {n} batches of epoch 0 of '{cfg.name}' through the whole path "
                      f"(schedule, sample, histogram, TopHot+fill, gather of {rows} rows); {dt:.1f} s on one thread",
            "phase_seconds": {k: round(v, 4) for k, v in phases.items()}, "host_cpus": os.cpu_count()}


def link_probe(workload, seed, dev):
    """Host-link rates, one JSON line: plain runtime copies pinned -> HBM (whole, in pieces, strided), one runtime copy per
    run of consecutive rows of the first batch's pull plan, and the library's pull kernels on the same plan with nothing
    beside them."""
    import numpy as np
    import torch
    import synth
    from paper_2505_10806_amd import binding as B
    from paper_2505_10806_amd.pipeline import EpochPipeline

    def best_ms(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1))
        return best
    out = {}
    src = torch.empty(1 << 28, dtype=torch.float32).pin_memory()
    src.normal_()
    dst = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    ms = best_ms(lambda: dst.copy_(src, non_blocking=True))
    out["runtime_copy_1GiB"] = {"ms": ms, "GBps": (1 << 30) / ms / 1e6}
    pieces = [(dst[i << 24:(i + 1) << 24], src[i << 24:(i + 1) << 24]) for i in range(16)]
    ms = best_ms(lambda: [d.copy_(s, non_blocking=True) for d, s in pieces])
    out["runtime_copy_16x64MiB"] = {"ms": ms, "GBps": (1 << 30) / ms / 1e6}
    s2, d2 = src.view(-1, 256), dst.view(-1, 256)
    half = s2.shape[0] // 2
    ms = best_ms(lambda: d2[:half].copy_(s2[::2], non_blocking=True))
    out["runtime_copy_every_other_1KiB_row"] = {"ms": ms, "GBps": half * 1024 / ms / 1e6}
    del src, dst, pieces, s2, d2
    torch.cuda.empty_cache()

    wl = synth.build_workload(workload, seed=seed, device=dev, keep_features=False)
    row_bytes = 4 * wl.cfg.feat_dim
    pipe = EpochPipeline(wl, device=dev, mirror_cache=False)
    pipe.precompute(0, pipe.batches_per_epoch)
    pipe.read_sizes()
    torch.cuda.synchronize()
    st = pipe.state
    off = st.plan.offsets.cpu().numpy()
    pairs = st.plan.list.cpu().numpy().reshape(-1, 2)
    runs = {}
    for b in (0, 1, 8, 32, 100, 200):
        if b < pipe.batches_per_epoch:
            seg = pairs[off[b]:off[b + 1]]
            n_runs = int(((np.diff(seg[:, 0]) != 1) | (np.diff(seg[:, 1]) != 1)).sum()) + 1 if len(seg) else 0
            runs[str(b)] = {"rows": int(len(seg)), "runs_of_consecutive_rows": n_runs}
    out["plan_segments"] = runs
    seg = pairs[off[0]:off[1]]
    brk = np.flatnonzero((np.diff(seg[:, 0]) != 1) | (np.diff(seg[:, 1]) != 1)) + 1
    starts, ends = np.concatenate([[0], brk]), np.concatenate([brk, [len(seg)]])
    n_run = min(20000, len(starts))
    rows_copied = int((ends[:n_run] - starts[:n_run]).sum())
    cache_rows, remote = st.cache.cache_rows, wl.remote_store
    t0 = time.perf_counter()
    for i in range(n_run):
        s0, r0, ln = int(seg[starts[i], 0]), int(seg[starts[i], 1]), int(ends[i] - starts[i])
        cache_rows[s0:s0 + ln].copy_(remote[r0:r0 + ln], non_blocking=True)
    t_issue = time.perf_counter() - t0
    torch.cuda.synchronize()
    t_all = time.perf_counter() - t0
    out["one_runtime_copy_per_run"] = {"runs": n_run, "rows": rows_copied, "issue_ms": t_issue * 1e3, "done_ms": t_all * 1e3,
                                       "GBps": rows_copied * row_bytes / t_all / 1e9}
    ctx = pipe.ctx
    ctx.profile_enable(True)
    ctx.profile_reset()
    for _ in range(3):
        ctx.prefetch_planned(st.plan, 0, st.cache, wl.remote_store, wl.cfg.feat_dim)
    torch.cuda.synchronize()
    ms, cnt = ctx.profile_read(B.RG_K_CACHE_FILL)
    out["pull_kernel_on_batch0_segment_alone"] = {"rows": int(len(seg)), "ms": ms / cnt, "GBps": len(seg) * row_bytes / (ms / cnt) / 1e6}
    cache2 = B.FeatureCache(wl.cfg.num_nodes, min(wl.capacity_rows, wl.n_remote), wl.stride, dev)
    ctx.profile_reset()
    ctx.build_cache(st.counts, wl.home, wl.remote_store, wl.cfg.feat_dim, cache2)
    torch.cuda.synchronize()
    ms, _ = ctx.profile_read(B.RG_K_CACHE_FILL)
    k = int(cache2.num_cached.item())
    out["bulk_fill_kernel_alone"] = {"rows": k, "ms": ms, "GBps": k * row_bytes / ms / 1e6}
    print(json.dumps({"link_probe": workload, "peak_GBps": HOSTLINK_PEAK_GBS, **out}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="mini-batches in the timed region (default: one epoch)")
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--reps", type=int, default=5, help="repetitions of the timed region, each from a cold cache (median reported)")
    ap.add_argument("--workload", default="stress")
    ap.add_argument("--seed", type=int, default=2025)
    ap.add_argument("--cpu-batches", type=int, default=None,
                    help="batches the CPU oracle is timed on (0 = skip; default: about 12 s of CPU work)")
    ap.add_argument("--one-stream", action="store_true", help="copy miss rows on the same stream as the HBM rows")
    ap.add_argument("--bulk-fill", action="store_true",
                    help="pull all cached rows in one go after TopHot instead of batch by batch ahead of the gathers")
    ap.add_argument("--sampler-streams", type=int, default=2, help="batches sampled side by side during the offline stage")
    ap.add_argument("--no-double-buffer", action="store_true",
                    help="with more than one epoch of steps: do not precompute epoch e+1 while epoch e is served")
    ap.add_argument("--consumer", choices=["none", "mean"], default="none",
                    help="reduce every batch's gathered rows with the mean aggregator over its outermost block, on its own stream")
    ap.add_argument("--queue-depth", type=int, default=3, help="output buffers the gathers may run ahead of the consumer")
    ap.add_argument("--no-plan", action="store_true",
                    help="prefetch with a claim pass over every batch instead of the per-epoch prefetch plan")
    ap.add_argument("--sample-group", type=int, default=8,
                    help="batches sampled by one rg_sample_blocks_group call")
    ap.add_argument("--histogram", choices=["epoch", "sampled", "batch"], default="epoch",
                    help="access counts from one LDS-privatised pass over the epoch's id lists, straight from the sampler's "
                         "membership bitmaps after every group, or one global-atomic pass per batch")
    ap.add_argument("--node-order", choices=["ascending", "first_seen"], default="ascending",
                    help="order of the nodes inside a tier of a block")
    ap.add_argument("--mirror-pulls", choices=("group", "batch"), default="group",
                    help="mirrored cache only: one pull per sampler call with its list read off the sampler's bitmaps, or one per batch")
    ap.add_argument("--pull-cus", type=int, default=16,
                    help="compute units reserved for the host-link pull kernels (0 = no split): their stream runs on these, every other stream on the rest")
    ap.add_argument("--coupled-misses", action="store_true",
                    help="fork to the miss stream and join back for every batch instead of letting the miss rows of consecutive batches follow each other")
    ap.add_argument("--no-mirror", action="store_true",
                    help="do not lay a cache that can hold the whole remote partition out as its mirror (rows are then pulled "
                         "after TopHot, from the prefetch plan, instead of while the batches are being sampled)")
    ap.add_argument("--keep-rows", action="store_true",
                    help="mirrored cache only: rows pulled in an earlier epoch stay resident instead of every epoch starting cold")
    ap.add_argument("--period-epochs", type=int, default=1,
                    help="epochs precomputed, counted and cached together (1: a cache per epoch from that epoch's counts; "
                         "E: one cache from the counts of E epochs, as Alg. 1 lines 1-4 read)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the extra passes (whole-epoch rate, gather kernel without concurrent pulls, hit curve)")
    ap.add_argument("--link-probe", action="store_true",
                    help="only measure the host link: runtime (SDMA) copies from pinned memory against the library's zero-copy "
                         "pull kernels on the workload's own pull plan")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy a few times (reference for hardware byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the remote partition is pinned host memory); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth
    from paper_2505_10806_amd import binding as B
    from paper_2505_10806_amd.pipeline import EpochPipeline

    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        dst.copy_(src)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(5):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        print(json.dumps({"copy_bytes_read": 1 << 30, "copy_bytes_written": 1 << 30, "ms": ms,
                          "GBps_read_plus_write": 2 * (1 << 30) / (ms * 1e-3) / 1e9}), flush=True)
        return
    if args.link_probe:
        link_probe(args.workload, args.seed, dev)
        return
    t_gen = time.perf_counter()
    wl = synth.build_workload(args.workload, seed=args.seed, device=dev)
    cfg = wl.cfg
    torch.cuda.synchronize()
    log(f"[bench] workload {cfg.name}: N={cfg.num_nodes} nnz={wl.nnz} D={cfg.feat_dim} fanouts={cfg.fanouts} "
        f"batch={cfg.batch_size} local={wl.n_local} remote={wl.n_remote} capacity={wl.capacity_rows} "
        f"(generated in {time.perf_counter() - t_gen:.1f} s)")

    bpe = wl.batches_per_epoch()
    per_period = bpe * max(1, args.period_epochs)
    steps = args.steps if args.steps is not None else per_period
    if steps % max(1, args.period_epochs):
        print("bench.py: --steps must be a multiple of --period-epochs", file=sys.stderr)
        sys.exit(2)
    warmup, reps = args.warmup, max(1, args.reps)
    row_bytes = 4 * cfg.feat_dim
    multi_epoch = steps > per_period
    def make_pipeline(prefetch):
        return EpochPipeline(wl, device=dev, two_streams=not args.one_stream, prefetch=prefetch,
                             sampler_streams=args.sampler_streams, double_buffer=(multi_epoch and not args.no_double_buffer),
                             planned_prefetch=not args.no_plan, sample_group=args.sample_group,
                             histogram=args.histogram, node_order=args.node_order, period_epochs=args.period_epochs,
                             mirror_cache=False if args.no_mirror else None, keep_rows=args.keep_rows, mirror_pulls=args.mirror_pulls,
                             pull_cus=args.pull_cus, decoupled_misses=not args.coupled_misses,
                             consumer=None if args.consumer == "none" else args.consumer,
                             queue_depth=args.queue_depth if args.consumer != "none" else 1)

    pipe = make_pipeline(not args.bulk_fill)
    # the gathers run on the stream this with-block makes current: one of the pipeline's own when it splits the compute units
    main_stream = pipe.work_stream or torch.cuda.Stream()
    with torch.cuda.stream(main_stream):
        ctx = pipe.ctx
        if warmup > 0:
            run_steps(pipe, warmup)
        times = timed_reps(pipe, steps, reps)
        prof_dt, prof, totals = profiled_pass(pipe, steps, dev)
        # the roofline's kernel in a pass of its own, the only kernel bracketed: brackets on every stream shift what runs beside what
        _, g_prof, g_totals = profiled_pass(pipe, steps, dev, only=[B.RG_K_GATHER_HBM])
        roof = gather_roofline(g_prof, g_totals, row_bytes)
        roof["avg_launch_ms_all_kernels_bracketed"] = gather_roofline(prof, totals, row_bytes)["avg_launch_ms"]

        # the offline stage alone (schedule, sampling, histogram, TopHot, plan), same batches, device idle otherwise
        offline_ms = None
        if not multi_epoch:
            ts = []
            for _ in range(3):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                pipe.precompute(0, min(steps, per_period) // pipe.period_epochs)
                torch.cuda.synchronize()
                ts.append((time.perf_counter() - t0) * 1e3)
            offline_ms = statistics.median(ts)

        full_epoch = None
        if not args.no_extras and steps != per_period and not multi_epoch and args.period_epochs == 1:
            run_steps(pipe, bpe)                                     # warm-up at the whole epoch's sizes
            full_times = timed_reps(pipe, bpe, 3)
            f_dt, f_prof, f_totals = profiled_pass(pipe, bpe, dev, only=[B.RG_K_GATHER_HBM])
            f_roof = gather_roofline(f_prof, f_totals, row_bytes)
            full_epoch = dict(spread(full_times, bpe), batches=bpe,
                              k_gather_hbm_frac=f_roof["frac"], k_gather_hbm_avg_launch_ms=f_roof["avg_launch_ms"])

    med = statistics.median(times)
    n_local, n_hit, n_miss = [int(x) for x in totals["stats"].cpu().tolist()]
    rows = totals["rows"]
    assert rows == n_local + n_hit + n_miss, "gather statistics do not add up"
    cached_rows = int(totals["cached"].item()) if not args.keep_rows else 0    # with kept rows fewer than the selected rows are pulled
    m_ms, _ = prof["gather_miss"]
    f_ms, _ = prof["cache_fill"]
    per_row_traffic, traffic_source = recorded_traffic(cfg.name)
    result = {
        "metric": "mini-batch sample+gather/sec; feature gather GB/s vs HBM peak; cache hit %",
        "value": steps / med,
        "unit": "batches/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": med * 1e3 / steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32 indices / fp32 rows (copy)",
        "data": "synthetic",
        "timing": dict(spread(times, steps),
                       step_definition=("one batch of a %d-batch epoch taken from a cold cache through schedule, sampling, histogram, "
                                        "TopHot, pulls and gather" % min(steps, bpe)) if not multi_epoch else
                                       "one batch of %d epochs run back to back with the double-buffered cache" % -(-steps // bpe),
                       profiled_pass_ms=prof_dt * 1e3, offline_stage_alone_ms=offline_ms,
                       note="value = steps / median; kernel durations come from the extra profiled pass"),
        "config": {"workload": cfg.name, "num_nodes": cfg.num_nodes, "nnz": wl.nnz, "feat_dim": cfg.feat_dim,
                   "fanouts": list(cfg.fanouts), "batch_size": cfg.batch_size, "batches_per_epoch": bpe,
                   "epochs_per_rep": totals["epochs"],
                   "cache_capacity_rows": wl.capacity_rows, "miss_stream": "shared" if args.one_stream else "separate",
                   "cache_fill": "bulk" if args.bulk_fill else ("pulled as the batches are sampled" if pipe.mirror else "prefetch by first use"),
                   "sampler_streams": args.sampler_streams, "sample_group": args.sample_group,
                   "double_buffered_cache": bool(multi_epoch and not args.no_double_buffer),
                   "planned_prefetch": pipe.planned, "consumer": args.consumer, "queue_depth": pipe.queue_depth,
                   "histogram": pipe.histogram, "node_order": args.node_order, "period_epochs": pipe.period_epochs,
                   "pull_cus": pipe.pull_cus, "decoupled_misses": pipe.decoupled, "mirrored_cache": pipe.mirror, "mirror_pulls": args.mirror_pulls if pipe.mirror else None, "rows_kept_across_epochs": pipe.keep_rows,
                   "GPU_MAX_HW_QUEUES": os.environ.get("GPU_MAX_HW_QUEUES"), "GPU_MAX_HW_QUEUES_set_by": "user" if HWQ_SET_BY_USER else "bench.py"},
        "roofline": {"bound": "hbm", "kernel": "k_gather_hbm", "achieved": roof["achieved"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": roof["frac"],
                     # not measured in this run: bytes per row from the recorded counter run, times this run's rows per launch
                     "traffic": per_row_traffic * roof["hbm_rows"] / max(roof["launches"], 1) if per_row_traffic else None,
                     "traffic_source": traffic_source,
                     "algorithmic_bytes_per_launch": roof["algorithmic_bytes_per_launch"],
                     "avg_launch_ms": roof["avg_launch_ms"], "launches": roof["launches"],
                     "avg_launch_ms_all_kernels_bracketed": roof["avg_launch_ms_all_kernels_bracketed"],
                     "timed_by": "hipEvents around each k_gather_hbm launch on its own stream, in a pass that brackets no other kernel",
                     "condition": "bulk fill: nothing runs beside the gathers" if args.bulk_fill
                                  else "host-link pulls of later batches run beside the gathers"},
        "gather": {"rows": rows, "n_local": n_local, "n_hit": n_hit, "n_miss": n_miss,
                   "cache_hit_pct": 100.0 * n_hit / max(1, n_hit + n_miss),
                   "payload_GBps_hbm_kernel": roof["achieved"] / 2,
                   "miss_hostlink_GBps": row_bytes * n_miss / (m_ms * 1e-3) / 1e9 if m_ms > 0 and n_miss else None,
                   "cache_fill_hostlink_GBps": row_bytes * cached_rows / (f_ms * 1e-3) / 1e9 if f_ms > 0 and cached_rows else None,
                   "cached_rows": cached_rows},
        "sampler": {"sampled_edges": int(totals["edges"].item()), "input_nodes": rows,
                    "sampled_edges_per_s_whole_path": int(totals["edges"].item()) / med,
                    "draw_kernel_edges_per_s": int(totals["edges"].item()) / (prof["sample"][0] * 1e-3) if prof["sample"][0] > 0 else None},
        "hostlink": {"bound": "pcie", "kernel": "k_prefetch_pull / k_cache_fill", "peak": HOSTLINK_PEAK_GBS, "unit": "GB/s",
                     "achieved": row_bytes * cached_rows / (f_ms * 1e-3) / 1e9 if f_ms > 0 and cached_rows else None,
                     "note": "sum of pull-kernel durations; the pulls run beside the gathers on their own stream"},
        "kernel_ms": {k: {"total_ms": v[0], "launches": v[1]} for k, v in prof.items()},
        # hits and misses of each epoch served in the profiled pass (with --period-epochs E, E epochs share one cache)
        "per_epoch": [{"n_local": int(a), "n_hit": int(b), "n_miss": int(c), "hit_pct": 100.0 * int(b) / max(1, int(b) + int(c))}
                      for a, b, c in (t.cpu().tolist() for t in totals["per_epoch"])],
    }
    if full_epoch is not None:
        result["full_epoch"] = full_epoch
    elif not multi_epoch and steps == per_period and args.period_epochs == 1:
        result["full_epoch"] = dict(spread(times, bpe), batches=bpe, k_gather_hbm_frac=roof["frac"],
                                    k_gather_hbm_avg_launch_ms=roof["avg_launch_ms"])

    if not args.no_extras:
        # requests for remote rows a cache of a given size would serve, from the last epoch's histogram (no cache is built)
        fracs = [0.01, 0.05, 0.10, 0.15, 0.20, 0.50, 1.00]
        caps = [int(f * wl.n_remote) for f in fracs] + [wl.capacity_rows]
        hits, total = ctx.cache_hit_curve(pipe.counts, wl.home, caps)
        torch.cuda.synchronize()
        total = int(total.item())
        hits, caps = hits[:-1], caps[:-1]
        result["cache_hit_curve"] = {"period": f"{pipe.n_batches} batches (last epoch run)", "remote_requests": total,
                                     "points": [{"capacity_frac_of_remote": f, "capacity_rows": c,
                                                 "hit_pct": 100.0 * int(h) / max(total, 1), "remote_fetches": total - int(h)}
                                                for f, c, h in zip(fracs, caps, hits.cpu().tolist())]}
        if not args.bulk_fill and not multi_epoch and args.period_epochs == 1:
            # the same gathers with all rows pulled beforehand: the copy kernel with nothing beside it
            n_b = min(steps, bpe)
            pipe.close()
            del pipe
            torch.cuda.empty_cache()
            bulk = make_pipeline(False)
            with torch.cuda.stream(bulk.work_stream or torch.cuda.Stream()):
                run_steps(bulk, n_b)
                _, b_prof, b_totals = profiled_pass(bulk, n_b, dev, only=[B.RG_K_GATHER_HBM])
            b_roof = gather_roofline(b_prof, b_totals, row_bytes)
            result["roofline"]["frac_without_concurrent_pulls"] = b_roof["frac"]
            result["roofline"]["avg_launch_ms_without_concurrent_pulls"] = b_roof["avg_launch_ms"]
            pipe = bulk
    a_ms, a_launches = prof["mean_aggregate"]
    if a_launches:
        result["consumer"] = {"kernel": "k_mean_aggregate", "total_ms": a_ms, "launches": a_launches}
    n_cpu = args.cpu_batches
    pipe.close()
    del pipe
    if n_cpu is None or n_cpu > 0:
        torch.cuda.empty_cache()
        log("[bench] timing the CPU oracle on a bounded sample ...")
        result["cpu_baseline"] = cpu_baseline(wl, n_cpu)
    print(json.dumps(result), flush=True)
    del wl
    B.close_shared_streams()


if __name__ == "__main__":
    main()
