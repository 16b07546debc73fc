#!/usr/bin/env python3
"""Benchmark of the RapidGNN data path on one MI355X.

A step is one mini-batch taken through the whole hot path: epoch schedule (once per epoch), k-hop
sampling, access histogram, TopHot + cache fill (once per epoch, amortised over its batches) and the
per-batch feature gather.  Inputs are synthetic (seeded Chung-Lu graph, N(0,1) features) and resident
in HBM / pinned host memory before the timed region starts.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

# The pipeline keeps up to five streams busy at once (gathers, miss rows, host-link pulls, two more sampler lanes);
# with HIP's default of 4 hardware queues two of them would share a queue and serialise.
if int(os.environ.get("GPU_MAX_HW_QUEUES", "0") or 0) < 8:
    os.environ["GPU_MAX_HW_QUEUES"] = "8"

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E peak
HOSTLINK_PEAK_GBS = 64.0   # PCIe Gen5 x16, one direction

# HBM bytes moved by one k_gather_hbm launch on the stress workload, measured with rocprofv3 --pmc (FETCH_SIZE and
# WRITE_SIZE, one counter per run, each scaled by what the same counter reads for a plain 1 GiB copy: x2.000 and
# x1.000).  The figures and the commands are in profiles/stress_gather_hbm_pmc_traffic.txt.
PMC_TRAFFIC = {"stress": {"fetch_kib": 404251.2, "fetch_scale": 2.0, "write_kib": 795996.3, "write_scale": 1.0,
                          "rows_per_launch": 795995}}


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def run_steps(pipe, steps, totals=None):
    """Run `steps` batches through the whole path, epoch after epoch (the last epoch may be partial)."""
    import torch
    marks = {"t": time.perf_counter()}

    def started(p, _k):                      # called once the epoch's offline stage has finished (host has its sizes)
        if totals is not None:
            now = time.perf_counter()
            totals["offline_s"] += now - marks["t"]
            marks["t"] = now

    def account(p, _k):
        if totals is not None:
            nb = p.n_batches
            totals["stats"] += p.stats[:nb].sum(0)
            totals["rows"] += sum(p.sizes[:nb])
            totals["edges"] += p.edge_counts[:nb].sum()
            totals["cached"] += p.cache.num_cached.clone()
            totals["epochs"] += 1
    full, rem = divmod(steps, pipe.max_batches)
    if full:
        pipe.run_epochs(0, full, pipe.max_batches, on_epoch_done=account, on_epoch_start=started)
    if rem:
        pipe.run_epochs(full, 1, rem, on_epoch_done=account, on_epoch_start=started)
    torch.cuda.current_stream().synchronize()


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="mini-batches in the timed region (default: one epoch)")
    ap.add_argument("--warmup", type=int, default=8)
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
    ap.add_argument("--early-pull", action="store_true",
                    help="pull rows into a staging area during the offline stage (only when the cache can hold every remote node)")
    ap.add_argument("--consumer", choices=["none", "mean"], default="none",
                    help="reduce every batch's gathered rows with the mean aggregator over its outermost block, on its own stream")
    ap.add_argument("--queue-depth", type=int, default=3, help="output buffers the gathers may run ahead of the consumer")
    ap.add_argument("--no-plan", action="store_true",
                    help="prefetch with a claim pass over every batch instead of the per-epoch prefetch plan")
    ap.add_argument("--sample-group", type=int, default=8,
                    help="batches sampled by one rg_sample_blocks_group call")
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
    t_gen = time.perf_counter()
    wl = synth.build_workload(args.workload, seed=args.seed, device=dev)
    cfg = wl.cfg
    torch.cuda.synchronize()
    log(f"[bench] workload {cfg.name}: N={cfg.num_nodes} nnz={wl.nnz} D={cfg.feat_dim} fanouts={cfg.fanouts} "
        f"batch={cfg.batch_size} local={wl.n_local} remote={wl.n_remote} capacity={wl.capacity_rows} "
        f"(generated in {time.perf_counter() - t_gen:.1f} s)")

    bpe = wl.batches_per_epoch()
    steps = args.steps if args.steps is not None else bpe
    warmup = args.warmup
    main_stream = torch.cuda.Stream()
    with torch.cuda.stream(main_stream):
        pipe = EpochPipeline(wl, device=dev, max_batches=min(max(steps, warmup, 1), bpe), two_streams=not args.one_stream,
                             prefetch=not args.bulk_fill, sampler_streams=args.sampler_streams,
                             double_buffer=(steps > bpe and not args.no_double_buffer), early_pull=args.early_pull, planned_prefetch=not args.no_plan, sample_group=args.sample_group,
                             consumer=None if args.consumer == "none" else args.consumer,
                             queue_depth=args.queue_depth if args.consumer != "none" else 1)
        ctx = pipe.ctx
        if warmup > 0:
            run_steps(pipe, warmup)
        totals = {"stats": torch.zeros(3, dtype=torch.int64, device=dev), "rows": 0,
                  "edges": torch.zeros((), dtype=torch.int64, device=dev),
                  "cached": torch.zeros(1, dtype=torch.int64, device=dev), "epochs": 0, "offline_s": 0.0}
        pipe.profile_enable(True)
        pipe.profile_reset()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(pipe, steps, totals)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        pipe.profile_enable(False)

    n_local, n_hit, n_miss = [int(x) for x in totals["stats"].cpu().tolist()]
    rows = totals["rows"]
    assert rows == n_local + n_hit + n_miss, "gather statistics do not add up"
    row_bytes = 4 * cfg.feat_dim
    prof = {name: pipe.profile_read(kid) for name, kid in
            [("gather_hbm", B.RG_K_GATHER_HBM), ("gather_miss", B.RG_K_GATHER_MISS), ("sample", B.RG_K_SAMPLE),
             ("histogram", B.RG_K_HISTOGRAM), ("cache_fill", B.RG_K_CACHE_FILL), ("mean_aggregate", B.RG_K_AGGREGATE)]}
    g_ms, g_launches = prof["gather_hbm"]
    hbm_rows = n_local + n_hit
    alg_bytes = 2.0 * row_bytes * hbm_rows                       # every HBM-served row is read once and written once
    achieved = alg_bytes / (g_ms * 1e-3) / 1e9 if g_ms > 0 else 0.0
    cached_rows = int(totals["cached"].item())
    m_ms, _ = prof["gather_miss"]
    f_ms, _ = prof["cache_fill"]
    traffic = None
    if cfg.name in PMC_TRAFFIC and g_launches:
        t = PMC_TRAFFIC[cfg.name]
        per_row = (t["fetch_kib"] * t["fetch_scale"] + t["write_kib"] * t["write_scale"]) * 1024.0 / t["rows_per_launch"]
        traffic = per_row * hbm_rows / g_launches            # measured bytes per row x rows per launch of this run
    result = {
        "metric": "mini-batch sample+gather/sec; feature gather GB/s vs HBM peak; cache hit %",
        "value": steps / dt,
        "unit": "batches/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": dt * 1e3 / steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32 indices / fp32 rows (copy)",
        "data": "synthetic",
        "config": {"workload": cfg.name, "num_nodes": cfg.num_nodes, "nnz": wl.nnz, "feat_dim": cfg.feat_dim,
                   "fanouts": list(cfg.fanouts), "batch_size": cfg.batch_size, "epochs_timed": totals["epochs"],
                   "cache_capacity_rows": wl.capacity_rows, "miss_stream": "shared" if args.one_stream else "separate",
                   "cache_fill": "bulk" if args.bulk_fill else "prefetch by first use",
                   "sampler_streams": args.sampler_streams, "sample_group": args.sample_group,
                   "double_buffered_cache": bool(steps > bpe and not args.no_double_buffer),
                   "early_pull": pipe.early_pull, "planned_prefetch": pipe.planned, "consumer": args.consumer,
                   "queue_depth": pipe.queue_depth},
        "roofline": {"bound": "hbm", "kernel": "k_gather_hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes_per_launch": alg_bytes / max(g_launches, 1),
                     "avg_launch_ms": g_ms / max(g_launches, 1), "launches": g_launches},
        "gather": {"rows": rows, "n_local": n_local, "n_hit": n_hit, "n_miss": n_miss,
                   "cache_hit_pct": 100.0 * n_hit / max(1, n_hit + n_miss),
                   "payload_GBps_hbm_kernel": row_bytes * hbm_rows / (g_ms * 1e-3) / 1e9 if g_ms > 0 else 0.0,
                   "miss_hostlink_GBps": row_bytes * n_miss / (m_ms * 1e-3) / 1e9 if m_ms > 0 and n_miss else None,
                   "cache_fill_hostlink_GBps": row_bytes * cached_rows / (f_ms * 1e-3) / 1e9 if f_ms > 0 and cached_rows else None,
                   "cached_rows": cached_rows},
        "sampler": {"sampled_edges": int(totals["edges"].item()), "input_nodes": rows,
                    "sampled_edges_per_s_whole_path": int(totals["edges"].item()) / dt,
                    "draw_kernel_edges_per_s": int(totals["edges"].item()) / (prof["sample"][0] * 1e-3) if prof["sample"][0] > 0 else None},
        "hostlink": {"bound": "pcie", "kernel": "k_prefetch_pull / k_cache_fill", "peak": HOSTLINK_PEAK_GBS, "unit": "GB/s",
                     "achieved": row_bytes * cached_rows / (f_ms * 1e-3) / 1e9 if f_ms > 0 and cached_rows else None,
                     "note": "sum of pull-kernel durations; the pulls run beside the gathers on their own stream"},
        "kernel_ms": {k: {"total_ms": v[0], "launches": v[1]} for k, v in prof.items()},
        # host clock: time until each epoch's offline stage (schedule, sampling, histogram, TopHot, plan) had finished,
        # and the rest (pulls and gathers); with double buffering the next epoch's offline stage hides in "online"
        "phase_ms": {"offline_until_sizes_known": totals["offline_s"] * 1e3, "online": (dt - totals["offline_s"]) * 1e3},
    }

    # requests for remote rows a cache of a given size would serve, from the last epoch's histogram (no cache is built)
    fracs = [0.01, 0.05, 0.10, 0.15, 0.20, 0.50, 1.00]
    caps = [int(f * wl.n_remote) for f in fracs] + [wl.capacity_rows]
    hits, total = ctx.cache_hit_curve(pipe.counts, wl.home, caps)
    torch.cuda.synchronize()
    total = int(total.item())
    predicted = int(hits[-1].item())
    hits, caps = hits[:-1], caps[:-1]
    result["gather"]["cache_hit_pct_predicted_from_histogram"] = 100.0 * predicted / max(total, 1)
    if totals["epochs"] == 1:      # one epoch: the hits counted by the gathers are exactly those the histogram predicts
        assert predicted == n_hit and total == n_hit + n_miss, "cache hits differ from the histogram's prediction"
    result["cache_hit_curve"] = {"period": f"{pipe.n_batches} batches (last timed epoch)", "remote_requests": total,
                                 "points": [{"capacity_frac_of_remote": f, "capacity_rows": c,
                                             "hit_pct": 100.0 * int(h) / max(total, 1), "remote_fetches": total - int(h)}
                                            for f, c, h in zip(fracs, caps, hits.cpu().tolist())]}
    a_ms, a_launches = prof["mean_aggregate"]
    if a_launches:
        # per launch: one feature row read per sampled edge of the outermost hop, one row written per destination
        last = pipe.H - 1
        e_last = sum(int(st.edge_counts[:st.n_batches, last].sum().item()) for st in pipe.states[:1]) if steps <= bpe else None
        result["consumer"] = {"kernel": "k_mean_aggregate", "total_ms": a_ms, "launches": a_launches,
                              "outermost_hop_edges": e_last,
                              "algorithmic_GBps": (row_bytes * (e_last + sum(int(x) for x in pipe.state.tier_offs[:pipe.n_batches, pipe.H].cpu().tolist()))
                                                   / (a_ms * 1e-3) / 1e9) if e_last else None}
    n_cpu = args.cpu_batches
    if n_cpu is None or n_cpu > 0:
        del pipe
        torch.cuda.empty_cache()
        log("[bench] timing the CPU oracle on a bounded sample ...")
        result["cpu_baseline"] = cpu_baseline(wl, n_cpu)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
