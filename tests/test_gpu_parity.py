"""Bit-exact parity of the HIP path (through the C ABI) against the CPU oracle: tolerance 0.

Everything on this path is integer, index or copy work, so every comparison is exact equality.
"""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_common import HipBatch, assert_batch_equal, host_graph, log, np_i64

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def B():
    from paper_2505_10806_amd import binding
    return binding


@pytest.fixture(scope="module")
def ctx(B):
    c = B.Context(0)
    yield c
    c.close()


def _i32(a):
    return torch.as_tensor(np.ascontiguousarray(a, dtype=np.int32), device=DEV)


# ------------------------------------------------------------------------------ schedule
@pytest.mark.parametrize("n", [1, 2, 7, 2047, 2048, 2049, 5000, 120_000])
def test_epoch_schedule(ctx, n):
    log(f"[schedule] n={n}")
    rng = np.random.default_rng(n)
    ids = rng.choice(max(4 * n, 16), size=n, replace=False).astype(np.int32)
    for seed, epoch in [(2025, 0), ((7 << 33) + 5, 3)]:
        got = ctx.epoch_schedule(_i32(ids), seed, epoch)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), oracle.epoch_schedule(ids, seed, epoch))


def test_epoch_schedule_empty(ctx):
    ctx.epoch_schedule(torch.empty(0, dtype=torch.int32, device=DEV), 1, 0)


# ------------------------------------------------------------------------------ sampler
def _run_blocks(B, ctx, csr, seeds_np, fanouts, seed, epoch, bufs=None, with_local=True, first_seen=False):
    if bufs is None:
        bufs = B.BlockBuffers(csr.num_nodes, csr.num_edges, max(len(seeds_np), 1), fanouts, DEV, with_local=with_local)
    if first_seen:      # the node order is a parameter of the group call
        seeds = _i32(seeds_np) if len(seeds_np) else torch.empty(0, dtype=torch.int32, device=DEV)
        ctx.sample_blocks_group(csr, [seeds], fanouts, seed, epoch, [bufs], node_order=B.RG_ORDER_FIRST_SEEN)
    else:
        ctx.sample_blocks(csr, _i32(seeds_np), len(seeds_np), fanouts, seed, epoch, bufs)
    return HipBatch(bufs, len(fanouts))


def _handmade_graph(n, p_dense, n_dense, p, rng):
    adj = [[] for _ in range(n)]
    for u in range(n):
        for v in range(u + 1, n):
            if rng.random() < (p_dense if u < n_dense else p):
                adj[u].append(v)
                adj[v].append(u)
    rp = np.zeros(n + 1, dtype=np.int64)
    rp[1:] = np.cumsum([len(a) for a in adj])
    ci = np.array([u for a in adj for u in sorted(a)], dtype=np.int32)
    return rp, ci


@pytest.mark.parametrize("first_seen", [False, True])
@pytest.mark.parametrize("rp_dtype", [torch.int32, torch.int64])
@pytest.mark.parametrize("fanouts", [(3, 2), (0, 4), (5,), (-1, 2), (-1, -1, -1), (64, 3), (100, 100), (1024,)])
def test_blocks_handmade_graph(B, ctx, fanouts, rp_dtype, first_seen):
    """Dense core (degrees up to ~400) so that large fan-outs still take the Floyd branch.  Both node orders."""
    log(f"[blocks handmade] fanouts={fanouts} rp={rp_dtype} first_seen={first_seen}")
    order = oracle.ORDER_FIRST_SEEN if first_seen else oracle.ORDER_ASCENDING
    rng = np.random.default_rng(17)
    rp, ci = _handmade_graph(500, 0.8, 40, 0.01, rng)
    csr = B.CsrGraph(torch.as_tensor(rp, device=DEV).to(rp_dtype), _i32(ci))
    seeds = np.array([3, 499, 41, 0, 250, 77], dtype=np.int32)
    for seed, epoch in [(5, 0), ((1 << 40) + 9, 7)]:
        hip = _run_blocks(B, ctx, csr, seeds, fanouts, seed, epoch, first_seen=first_seen)
        orc = oracle.sample_blocks(rp, ci, seeds, fanouts, seed, epoch, order)
        assert_batch_equal(hip, orc, len(fanouts), f"seed={seed} epoch={epoch}")


def test_blocks_on_generated_csr(B, ctx):
    """Randomised: arbitrary CSR rows (repeated neighbours, self loops, empty rows), random distinct seeds, fan-outs
    that exercise the whole-row branch, both draw kernels and "all neighbours", both offset widths."""
    from hypothesis import HealthCheck, given, settings, strategies as st

    @st.composite
    def case(draw):
        n = draw(st.integers(1, 60))
        rows = [draw(st.lists(st.integers(0, n - 1), max_size=draw(st.sampled_from([0, 3, 8, 45])))) for _ in range(n)]
        seeds = draw(st.lists(st.integers(0, n - 1), max_size=min(n, 12), unique=True))
        fanouts = tuple(draw(st.lists(st.sampled_from([-1, 0, 1, 2, 5, 8, 9, 16, 17, 32, 33, 40]), min_size=1, max_size=3)))
        return (rows, seeds, fanouts, draw(st.integers(0, 2 ** 64 - 1)), draw(st.integers(0, 2 ** 32 - 1)), draw(st.booleans()),
                draw(st.booleans()))

    @settings(max_examples=120, deadline=None, derandomize=True, suppress_health_check=list(HealthCheck))
    @given(case())
    def run(c):
        rows, seeds, fanouts, seed, epoch, wide, first_seen = c
        rp = np.zeros(len(rows) + 1, dtype=np.int64)
        rp[1:] = np.cumsum([len(r) for r in rows])
        ci = np.array([u for r in rows for u in r], dtype=np.int32)
        csr = B.CsrGraph(torch.as_tensor(rp, device=DEV).to(torch.int64 if wide else torch.int32),
                         _i32(ci) if ci.size else torch.empty(0, dtype=torch.int32, device=DEV))
        hip = _run_blocks(B, ctx, csr, np.array(seeds, dtype=np.int32), fanouts, seed, epoch, first_seen=first_seen)
        orc = oracle.sample_blocks(rp, ci, np.array(seeds, dtype=np.int32), fanouts, seed, epoch,
                                   oracle.ORDER_FIRST_SEEN if first_seen else oracle.ORDER_ASCENDING)
        assert_batch_equal(hip, orc, len(fanouts), f"fanouts={fanouts} seeds={seeds} first_seen={first_seen}")

    run()


@pytest.mark.parametrize("first_seen", [False, True])
@pytest.mark.parametrize("group", [1, 2, 3, 8, 16])
@pytest.mark.parametrize("fanouts", [(5, 3), (40, 2), (-1, 4)])
def test_blocks_group_equals_separate_batches(B, ctx, group, fanouts, first_seen):
    """One call for several batches (different seed counts, one of them empty) gives each batch exactly the block
    of a call of its own; a smaller group after a larger one on the same context is unaffected by the earlier run."""
    log(f"[blocks group] group={group} fanouts={fanouts} first_seen={first_seen}")
    order = oracle.ORDER_FIRST_SEEN if first_seen else oracle.ORDER_ASCENDING
    rng = np.random.default_rng(group * 10 + len(fanouts))
    rp, ci = _handmade_graph(700, 0.7, 35, 0.015, rng)
    csr = B.CsrGraph(torch.as_tensor(rp, device=DEV), _i32(ci))
    sizes = [64, 0, 200, 1, 37, 128, 5, 90, 17, 300, 2, 64, 9, 111, 40, 256][:group]
    seeds_np = [rng.choice(700, size=n, replace=False).astype(np.int32) for n in sizes]
    outs = [B.BlockBuffers(700, ci.size, max(n, 1), fanouts, DEV) for n in sizes]
    ctx.sample_blocks_group(csr, [_i32(x) if x.size else torch.empty(0, dtype=torch.int32, device=DEV) for x in seeds_np],
                            fanouts, 99, 4, outs, node_order=B.RG_ORDER_FIRST_SEEN if first_seen else B.RG_ORDER_ASCENDING)
    # the group's membership bitmaps as access counts, with the first batch that names each node
    counts = torch.zeros(700, dtype=torch.int32, device=DEV)
    first = torch.full((700,), -1, dtype=torch.int32, device=DEV)
    ctx.access_histogram_sampled(group, counts, batch_index=range(10, 10 + group), first_batch=first)
    counts_orc = np.zeros(700, dtype=np.uint32)
    first_orc = np.full(700, 0xFFFFFFFF, dtype=np.uint32)
    for g in range(group):
        hip = HipBatch(outs[g], len(fanouts))
        orc = oracle.sample_blocks(rp, ci, seeds_np[g], fanouts, 99, 4, order)
        assert_batch_equal(hip, orc, len(fanouts), f"batch {g} of {group}")
        oracle.access_histogram(orc.input_nodes, counts_orc)
        first_orc[orc.input_nodes] = np.minimum(first_orc[orc.input_nodes], 10 + g)
    assert np.array_equal(counts.cpu().numpy().view(np.uint32), counts_orc), "counts from the membership bitmaps"
    assert np.array_equal(first.cpu().numpy().view(np.uint32), first_orc), "first batch from the membership bitmaps"
    with pytest.raises(B.RgError) as e:                    # a group size that is not the sampled one is refused
        ctx.access_histogram_sampled(group % 16 + 1, counts)
    assert e.value.status == B.RG_ERR_STATE
    # a single batch afterwards on the same context
    hip = _run_blocks(B, ctx, csr, seeds_np[0], fanouts, 7, 1, first_seen=first_seen)
    orc = oracle.sample_blocks(rp, ci, seeds_np[0], fanouts, 7, 1, order)
    assert_batch_equal(hip, orc, len(fanouts), "single batch after the group")


def test_blocks_degenerate_inputs(B, ctx):
    log("[blocks degenerate]")
    rp = np.array([0, 0, 1, 2, 2], dtype=np.int64)          # 0 and 3 isolated, 1 <-> 2
    ci = np.array([2, 1], dtype=np.int32)
    csr = B.CsrGraph(torch.as_tensor(rp, device=DEV).to(torch.int32), _i32(ci))
    for seeds in ([0], [], [1], [3, 0], [2, 1, 0, 3]):
        seeds = np.array(seeds, dtype=np.int32)
        hip = _run_blocks(B, ctx, csr, seeds, (4, 4), 1, 0)
        orc = oracle.sample_blocks(rp, ci, seeds, (4, 4), 1, 0)
        assert_batch_equal(hip, orc, 2, f"seeds={seeds.tolist()}")
    # a graph without edges
    rp0 = np.zeros(6, dtype=np.int64)
    csr0 = B.CsrGraph(torch.as_tensor(rp0, device=DEV), torch.empty(0, dtype=torch.int32, device=DEV))
    hip = _run_blocks(B, ctx, csr0, np.array([4, 1], dtype=np.int32), (3,), 1, 0)
    orc = oracle.sample_blocks(rp0, np.empty(0, dtype=np.int32), [4, 1], (3,), 1, 0)
    assert_batch_equal(hip, orc, 1, "edgeless")


def test_blocks_without_relabelling(B, ctx):
    rng = np.random.default_rng(3)
    rp, ci = _handmade_graph(300, 0.5, 10, 0.02, rng)
    csr = B.CsrGraph(torch.as_tensor(rp, device=DEV), _i32(ci))
    seeds = np.arange(0, 300, 7, dtype=np.int32)
    hip = _run_blocks(B, ctx, csr, seeds, (4, 3), 9, 1, with_local=False)
    orc = oracle.sample_blocks(rp, ci, seeds, (4, 3), 9, 1)
    assert_batch_equal(hip, orc, 2)


# ------------------------------------------------------------------------------ whole path
def _full_path(B, ctx, name, two_streams, device_counts):
    """Every batch of every epoch of a named workload: sample, histogram, TopHot + fill, gather."""
    wl = synth.build_workload(name, seed=2025, device=DEV)
    cfg = wl.cfg
    log(f"[full path] {name}: N={cfg.num_nodes} nnz={wl.nnz} D={cfg.feat_dim} capacity={wl.capacity_rows}")
    rp, ci = host_graph(wl)
    X = wl.features.cpu().numpy()
    home_np = wl.home.cpu().numpy()
    train_np = wl.train_ids.cpu().numpy()
    csr = B.CsrGraph(wl.row_ptr, wl.col_idx)
    H = len(cfg.fanouts)
    bufs = B.BlockBuffers(cfg.num_nodes, wl.nnz, cfg.batch_size, cfg.fanouts, DEV)
    cap_alloc = min(wl.capacity_rows, wl.n_remote)
    cache = B.FeatureCache(cfg.num_nodes, cap_alloc, wl.stride, DEV)
    out = torch.empty(bufs.frontier_ub[H], wl.stride, dtype=torch.float32, device=DEV)
    stats = torch.zeros(3, dtype=torch.int64, device=DEV)
    side = torch.cuda.Stream() if two_streams else None
    n_batches = wl.batches_per_epoch()
    for epoch in range(cfg.epochs):
        order = ctx.epoch_schedule(wl.train_ids, wl.seed, epoch)
        torch.cuda.synchronize()
        orc_batches = oracle.epoch_batches(train_np, cfg.batch_size, wl.seed, epoch, cfg.max_batches)
        assert len(orc_batches) == n_batches
        assert np.array_equal(order.cpu().numpy()[:sum(len(b) for b in orc_batches)], np.concatenate(orc_batches))
        counts = torch.zeros(cfg.num_nodes, dtype=torch.int32, device=DEV)
        counts_orc = np.zeros(cfg.num_nodes, dtype=np.uint32)
        hip_inputs, orc_inputs = [], []
        for b in range(n_batches):
            seeds = order[b * cfg.batch_size:(b + 1) * cfg.batch_size]
            ctx.sample_blocks(csr, seeds, seeds.numel(), cfg.fanouts, wl.seed, epoch, bufs)
            if device_counts:        # count stays on the device, no synchronisation before the histogram
                ctx.access_histogram(bufs.nodes, bufs.frontier_ub[H], counts, n_dev=bufs.tier_off[H + 1:])
            hip = HipBatch(bufs, H)
            if not device_counts:
                ctx.access_histogram(bufs.nodes, hip.nodes.size, counts)
            orc = oracle.sample_blocks(rp, ci, orc_batches[b], cfg.fanouts, wl.seed, epoch)
            assert_batch_equal(hip, orc, H, f"{name} epoch {epoch} batch {b}")
            oracle.access_histogram(orc.input_nodes, counts_orc)
            hip_inputs.append(bufs.nodes[:hip.nodes.size].clone())
            orc_inputs.append(orc.input_nodes)
        torch.cuda.synchronize()
        assert np.array_equal(counts.cpu().numpy().view(np.uint32), counts_orc), "histogram"
        # TopHot + VectorPull for this epoch's counts
        ctx.build_cache(counts, wl.home, wl.remote_store, cfg.feat_dim, cache)
        torch.cuda.synchronize()
        ids_orc, loc_orc = oracle.build_cache(counts_orc, home_np, wl.capacity_rows)
        k = int(cache.num_cached.item())
        assert k == ids_orc.size
        assert np.array_equal(cache.cache_ids[:k].cpu().numpy(), ids_orc), "cache_ids"
        assert np.array_equal(cache.loc.cpu().numpy(), loc_orc), "loc"
        rows_orc = oracle.fill_cache(X, ids_orc, wl.stride)
        assert np.array_equal(cache.cache_rows[:k, :cfg.feat_dim].cpu().numpy(), rows_orc[:, :cfg.feat_dim]), "cache rows"
        # per-batch feature assembly
        tot = np.zeros(3, dtype=np.int64)
        for b in range(n_batches):
            n = hip_inputs[b].numel()
            out.fill_(float("nan"))
            ctx.gather_features(hip_inputs[b], n, cache, wl.local_store, wl.remote_store, cfg.feat_dim, out, stats,
                                miss_stream=side)
            torch.cuda.synchronize()
            want, st_orc = oracle.gather_features(X, orc_inputs[b], loc_orc, wl.stride)
            assert np.array_equal(out[:n, :cfg.feat_dim].cpu().numpy(), want[:, :cfg.feat_dim]), f"gather batch {b}"
            assert tuple(stats.cpu().tolist()) == st_orc
            tot += np.array(st_orc)
        remote = (home_np.astype(np.int64) & 0xFFFFFFFF) >> 30 == 2
        assert tot[1] == int(counts_orc[ids_orc].sum())                  # hit count predicted by the histogram
        assert tot[1] + tot[2] == int(counts_orc[remote].sum())
        log(f"[full path] {name} epoch {epoch}: batches={n_batches} cached={k} "
            f"hit%={100.0 * tot[1] / max(1, tot[1] + tot[2]):.2f} rows={tot.sum()}")


def test_full_path_tiny(B, ctx):
    _full_path(B, ctx, "tiny", two_streams=False, device_counts=False)


def test_full_path_tiny_two_streams_device_counts(B, ctx):
    _full_path(B, ctx, "tiny", two_streams=True, device_counts=True)


def test_full_path_small(B, ctx):
    _full_path(B, ctx, "small", two_streams=True, device_counts=True)


@pytest.mark.parametrize("planned", [False, True])
def test_prefetch_by_first_use_matches_bulk_fill(B, ctx, planned):
    """Select-only TopHot followed by per-batch prefetch pulls each selected row exactly when a batch first
    needs it; gathers and the final cache contents equal those of the bulk pull."""
    wl = synth.build_workload("tiny", seed=11, device=DEV)
    cfg = wl.cfg
    H = len(cfg.fanouts)
    rp, ci = host_graph(wl)
    X = wl.features.cpu().numpy()
    home_np = wl.home.cpu().numpy()
    csr = B.CsrGraph(wl.row_ptr, wl.col_idx)
    bufs = B.BlockBuffers(cfg.num_nodes, wl.nnz, cfg.batch_size, cfg.fanouts, DEV)
    order = ctx.epoch_schedule(wl.train_ids, wl.seed, 0)
    torch.cuda.synchronize()
    orc_batches = oracle.epoch_batches(wl.train_ids.cpu().numpy(), cfg.batch_size, wl.seed, 0, 4)
    counts = torch.zeros(cfg.num_nodes, dtype=torch.int32, device=DEV)
    counts_orc = np.zeros(cfg.num_nodes, dtype=np.uint32)
    inputs_dev, inputs_orc = [], []
    for b in range(4):
        seeds = order[b * cfg.batch_size:(b + 1) * cfg.batch_size]
        ctx.sample_blocks(csr, seeds, seeds.numel(), cfg.fanouts, wl.seed, 0, bufs)
        torch.cuda.synchronize()
        n = int(bufs.tier_off[H + 1].item())
        inputs_dev.append(bufs.nodes[:n].clone())
        ctx.access_histogram(inputs_dev[-1], n, counts)
        orc = oracle.sample_blocks(rp, ci, orc_batches[b], cfg.fanouts, wl.seed, 0)
        oracle.access_histogram(orc.input_nodes, counts_orc)
        inputs_orc.append(orc.input_nodes)
    cache = B.FeatureCache(cfg.num_nodes, wl.capacity_rows, wl.stride, DEV)
    cache.cache_rows.fill_(float("nan"))
    cache.filled.fill_(-1)                                            # stale bits must be cleared by the select
    ctx.build_cache(counts, wl.home, None, cfg.feat_dim, cache)       # select only
    torch.cuda.synchronize()
    ids_orc, loc_orc = oracle.build_cache(counts_orc, home_np, wl.capacity_rows)
    k = ids_orc.size
    assert int(cache.num_cached.item()) == k and np.array_equal(cache.cache_ids[:k].cpu().numpy(), ids_orc)
    assert not cache.filled.cpu().numpy().any()
    assert torch.isnan(cache.cache_rows).all()
    slot_of = {int(v): s for s, v in enumerate(ids_orc)}
    resident = np.zeros(k, dtype=bool)
    out = torch.empty(bufs.frontier_ub[H], wl.stride, device=DEV)
    stats = torch.zeros(3, dtype=torch.int64, device=DEV)
    side = torch.cuda.Stream()
    if planned:
        # per-epoch plan: first batch of every node from the epoch histogram, slots grouped by it
        arena = torch.zeros(4, bufs.frontier_ub[H], dtype=torch.int32, device=DEV)
        tier_offs = torch.zeros(4, H + 2, dtype=torch.int32, device=DEV)
        for b in range(4):
            blk = oracle.sample_blocks(rp, ci, orc_batches[b], cfg.fanouts, wl.seed, 0)
            assert np.array_equal(inputs_dev[b].cpu().numpy(), blk.input_nodes)
            arena[b, :inputs_dev[b].numel()] = inputs_dev[b]
            tier_offs[b] = torch.as_tensor(blk.tier_off.astype(np.int32))
        first = torch.full((cfg.num_nodes,), -1, dtype=torch.int32, device=DEV)
        scratch_counts = torch.zeros_like(counts)
        ctx.access_histogram_epoch(arena, tier_offs, 4, H, cfg.batch_size, scratch_counts, first_batch=first)
        plan = B.PrefetchPlan(wl.capacity_rows, 4, DEV)
        ctx.plan_prefetch(cache, wl.home, first, plan)
        torch.cuda.synchronize()
        assert np.array_equal(scratch_counts.cpu().numpy().view(np.uint32), counts_orc)
        offs = plan.offsets.cpu().numpy()
        assert offs[0] == 0 and offs[5] == k and np.all(np.diff(offs[:6]) >= 0) and offs[4] == k   # every slot is used by some batch
    for b in range(4):
        n = inputs_dev[b].numel()
        if planned:
            ctx.prefetch_planned(plan, b, cache, wl.remote_store, cfg.feat_dim, stream=side)
        else:
            ctx.prefetch_cache_rows(inputs_dev[b], n, cache, wl.home, wl.remote_store, cfg.feat_dim, stream=side)
        side.synchronize()
        for v in inputs_orc[b]:
            if int(v) in slot_of:
                resident[slot_of[int(v)]] = True
        bits = np.unpackbits(cache.filled.cpu().numpy().view(np.uint8), bitorder="little")[:k].astype(bool)
        assert np.array_equal(bits, resident), f"resident set after batch {b}"
        rows = cache.cache_rows[:k, :cfg.feat_dim].cpu().numpy()
        assert np.array_equal(rows[resident], X[ids_orc[resident]])
        assert np.isnan(rows[~resident]).all()                        # nothing pulled before its first use
        ctx.gather_features(inputs_dev[b], n, cache, wl.local_store, wl.remote_store, cfg.feat_dim, out, stats)
        torch.cuda.synchronize()
        want, st = oracle.gather_features(X, inputs_orc[b], loc_orc)
        assert np.array_equal(out[:n, :cfg.feat_dim].cpu().numpy(), want)
        assert tuple(stats.cpu().tolist()) == st
    assert resident.all()
    # a second pass pulls nothing (every slot is resident)
    cache.cache_rows.fill_(0)
    ctx.prefetch_cache_rows(inputs_dev[0], inputs_dev[0].numel(), cache, wl.home, wl.remote_store, cfg.feat_dim)
    torch.cuda.synchronize()
    assert not cache.cache_rows.any()


def test_mirrored_cache_is_filled_before_tophot(B, ctx):
    """A cache that can hold the whole remote partition, laid out as its mirror: each batch's remote rows are pulled right
    after the batch is sampled (no TopHot result needed), TopHot then selects exactly the nodes that were pulled, and
    the gathers read a cached node's row at its remote-store row.  Rows, statistics and selection against the oracle;
    a second period keeps the resident rows and pulls only rows it is the first to name."""
    wl = synth.build_workload("tiny", seed=21, device=DEV)
    cfg, H = wl.cfg, len(wl.cfg.fanouts)
    rp, ci = host_graph(wl)
    X = wl.features.cpu().numpy()
    home_np = wl.home.cpu().numpy()
    csr = B.CsrGraph(wl.row_ptr, wl.col_idx)
    cache = B.FeatureCache(cfg.num_nodes, wl.n_remote, wl.stride, DEV, mirror_rows=wl.n_remote, home=wl.home)
    cache.cache_rows.fill_(float("nan"))
    with pytest.raises(B.RgError):                       # a mirror is never filled in bulk
        ctx.build_cache(torch.zeros(cfg.num_nodes, dtype=torch.int32, device=DEV), wl.home, wl.remote_store, cfg.feat_dim, cache)
    out = torch.empty(cfg.num_nodes, wl.stride, device=DEV)
    stats = torch.zeros(3, dtype=torch.int64, device=DEV)
    pulled_before = 0
    for epoch in (0, 1):
        order = ctx.epoch_schedule(wl.train_ids, wl.seed, epoch)
        counts = torch.zeros(cfg.num_nodes, dtype=torch.int32, device=DEV)
        counts_orc = np.zeros(cfg.num_nodes, dtype=np.uint32)
        inputs, inputs_dev = [], []
        for b in range(4):
            bufs = B.BlockBuffers(cfg.num_nodes, wl.nnz, cfg.batch_size, cfg.fanouts, DEV)
            seeds = order[b * cfg.batch_size:(b + 1) * cfg.batch_size]
            ctx.sample_blocks(csr, seeds, seeds.numel(), cfg.fanouts, wl.seed, epoch, bufs)
            ctx.access_histogram(bufs.nodes, bufs.frontier_ub[H], counts, n_dev=bufs.tier_off[H + 1:])
            # the batch's remote rows cross the link now, before any selection exists
            ctx.prefetch_cache_rows(bufs.nodes, bufs.frontier_ub[H], cache, wl.home, wl.remote_store, cfg.feat_dim,
                                    n_dev=bufs.tier_off[H + 1:])
            torch.cuda.synchronize()
            n = int(bufs.tier_off[H + 1].item())
            inputs_dev.append(bufs.nodes[:n].clone())
            orc = oracle.sample_blocks(rp, ci, seeds.cpu().numpy(), cfg.fanouts, wl.seed, epoch)
            assert np.array_equal(inputs_dev[-1].cpu().numpy(), orc.input_nodes)
            oracle.access_histogram(orc.input_nodes, counts_orc)
            inputs.append(orc.input_nodes)
        ctx.build_cache(counts, wl.home, None, cfg.feat_dim, cache)
        torch.cuda.synchronize()
        ids_orc, loc_orc = oracle.build_cache(counts_orc, home_np, wl.n_remote)
        k = int(cache.num_cached.item())
        assert k == ids_orc.size and np.array_equal(cache.cache_ids[:k].cpu().numpy(), ids_orc)
        assert np.array_equal(cache.loc.cpu().numpy(), loc_orc)
        # resident rows = every remote row named so far, each at its remote-store row; nothing else was written
        bits = np.unpackbits(cache.filled.cpu().numpy().view(np.uint8), bitorder="little")[:wl.n_remote]
        rows_now = (home_np[ids_orc].astype(np.int64) & 0x3FFFFFFF)
        assert bits[rows_now].all()
        resident = np.flatnonzero(bits)
        got = cache.cache_rows.cpu().numpy()
        remote_ids = np.flatnonzero(((home_np.astype(np.int64) & 0xFFFFFFFF) >> 30) == 2)
        assert np.array_equal(got[resident, :cfg.feat_dim], X[remote_ids[resident]])
        assert np.isnan(got[np.flatnonzero(bits == 0)]).all()
        if epoch == 0:
            assert resident.size == k
            pulled_before = resident.size
        else:
            assert pulled_before < resident.size < pulled_before + k      # only rows no earlier batch had named were pulled
        for b in range(4):
            ctx.gather_features(inputs_dev[b], inputs_dev[b].numel(), cache, wl.local_store, wl.remote_store, cfg.feat_dim, out, stats)
            torch.cuda.synchronize()
            want, st = oracle.gather_features(X, inputs[b], loc_orc)
            assert st[2] == 0 and tuple(stats.cpu().tolist()) == st
            assert np.array_equal(out[:inputs[b].size, :cfg.feat_dim].cpu().numpy(), want)
    with pytest.raises(B.RgError):                       # the plan made from TopHot's selection does not apply to a mirror
        ctx.plan_prefetch(cache, wl.home, torch.zeros(cfg.num_nodes, dtype=torch.int32, device=DEV), B.PrefetchPlan(wl.n_remote, 4, DEV))


def test_plan_segments_from_sampler_bitmaps(B, ctx):
    """rg_plan_sampled on a mirrored cache: after each sampler call the plan gains one segment = the remote rows the
    call's batches are the first to name, ascending, each paired with itself; rg_prefetch_planned pulls exactly those.
    Expected segments come from the oracle's input-node lists."""
    wl = synth.build_workload("tiny", seed=33, device=DEV)
    cfg, H = wl.cfg, len(wl.cfg.fanouts)
    rp, ci = host_graph(wl)
    X = wl.features.cpu().numpy()
    home_np = wl.home.cpu().numpy().astype(np.int64) & 0xFFFFFFFF
    csr = B.CsrGraph(wl.row_ptr, wl.col_idx)
    cache = B.FeatureCache(cfg.num_nodes, wl.n_remote, wl.stride, DEV, mirror_rows=wl.n_remote, home=wl.home)
    cache.cache_rows.fill_(float("nan"))
    cache.filled.zero_()
    groups = [3, 1, 4, 2]
    plan = B.PrefetchPlan(wl.n_remote, len(groups), DEV)
    plan.set_num_batches(len(groups))
    claimed = torch.zeros((cfg.num_nodes + 31) // 32, dtype=torch.int32, device=DEV)
    order = ctx.epoch_schedule(wl.train_ids, wl.seed, 0)
    order_np = order.cpu().numpy()
    seen = np.zeros(cfg.num_nodes, dtype=bool)
    b0, start = 0, 0
    remote_ids = np.flatnonzero((home_np >> 30) == 2)
    for seg, g in enumerate(groups):
        bufs = [B.BlockBuffers(cfg.num_nodes, wl.nnz, cfg.batch_size, cfg.fanouts, DEV) for _ in range(g)]
        seeds = [order[(b0 + j) * cfg.batch_size:(b0 + j + 1) * cfg.batch_size] for j in range(g)]
        ctx.sample_blocks_group(csr, seeds, cfg.fanouts, wl.seed, 0, bufs)
        with pytest.raises(B.RgError):                   # the call must name the group the context sampled last
            ctx.plan_sampled(g + 1, cache, claimed, plan, seg)
        ctx.plan_sampled(g, cache, claimed, plan, seg)
        ctx.prefetch_planned(plan, seg, cache, wl.remote_store, cfg.feat_dim)
        torch.cuda.synchronize()
        new = np.zeros(cfg.num_nodes, dtype=bool)
        for j in range(g):
            sd = order_np[(b0 + j) * cfg.batch_size:(b0 + j + 1) * cfg.batch_size]
            new[oracle.sample_blocks(rp, ci, sd, cfg.fanouts, wl.seed, 0).input_nodes] = True
        new &= ~seen
        seen |= new
        ids = np.flatnonzero(new & ((home_np >> 30) == 2))
        rows = home_np[ids] & 0x3FFFFFFF
        offs = plan.offsets.cpu().numpy()
        assert offs[seg] == start and offs[seg + 1] == start + rows.size, (seg, offs[:seg + 2], rows.size)
        pairs = plan.list.cpu().numpy()[2 * start:2 * (start + rows.size)].reshape(-1, 2)
        assert np.array_equal(pairs[:, 0], rows) and np.array_equal(pairs[:, 1], rows)
        start += rows.size
        b0 += g
        # the claim bitmap = every node named so far; resident rows = every remote row named so far
        cl = np.unpackbits(claimed.cpu().numpy().view(np.uint8), bitorder="little")[:cfg.num_nodes].astype(bool)
        assert np.array_equal(cl, seen)
        bits = np.unpackbits(cache.filled.cpu().numpy().view(np.uint8), bitorder="little")[:wl.n_remote].astype(bool)
        assert np.array_equal(bits, seen[remote_ids])
        got = cache.cache_rows.cpu().numpy()
        assert np.array_equal(got[bits, :cfg.feat_dim], X[remote_ids[bits]]) and np.isnan(got[~bits]).all()
    assert start > 0
    # argument checks: not a mirror, segment out of range, list too short
    plain = B.FeatureCache(cfg.num_nodes, wl.n_remote, wl.stride, DEV)
    for bad in (lambda: ctx.plan_sampled(groups[-1], plain, claimed, plan, 0),
                lambda: ctx.plan_sampled(groups[-1], cache, claimed, plan, len(groups)),
                lambda: ctx.plan_sampled(groups[-1], cache, claimed, B.PrefetchPlan(max(wl.n_remote - 1, 0), 4, DEV), 0)):
        with pytest.raises(B.RgError):
            bad()


@pytest.mark.parametrize("first_seen", [False, True])
@pytest.mark.parametrize("n_nodes,group", [(33, 1), (33, 5), (700, 16), (70_001, 3), (70_001, 8)])
def test_plan_segments_ragged_sizes(B, ctx, n_nodes, group, first_seen):
    """rg_plan_sampled where the bitmaps end inside a word, span one or several 1024-word blocks and a ragged last one,
    for groups of 1 to 16 batches (one of them empty) in either node order; home words drawn at random.  Two calls:
    the second segment holds only what the first has not claimed."""
    log(f"[plan ragged] N={n_nodes} group={group} first_seen={first_seen}")
    rng = np.random.default_rng(n_nodes + group)
    if n_nodes <= 1000:
        rp, ci = _handmade_graph(n_nodes, 0.5, min(8, n_nodes), 0.02 if n_nodes > 100 else 0.2, rng)
    else:
        rp_t, ci_t = synth.chung_lu_csr(n_nodes, 12, 2.3, seed=3)
        rp, ci = rp_t.numpy().astype(np.int64), ci_t.numpy()
    csr = B.CsrGraph(torch.as_tensor(rp, device=DEV), _i32(ci))
    remote = rng.random(n_nodes) < 0.6
    remote[rng.integers(n_nodes)] = True
    home_np = np.where(remote, (2 << 30) | (np.cumsum(remote) - 1), np.cumsum(~remote) - 1).astype(np.int64)
    home = torch.as_tensor(home_np.astype(np.uint32).view(np.int32), device=DEV)
    n_remote = int(remote.sum())
    cache = B.FeatureCache(n_nodes, n_remote, 4, DEV, mirror_rows=n_remote, home=home)
    plan = B.PrefetchPlan(n_remote, 2, DEV)
    plan.set_num_batches(2)
    claimed = torch.zeros((n_nodes + 31) // 32, dtype=torch.int32, device=DEV)
    fanouts = (4, 3)
    order = oracle.ORDER_FIRST_SEEN if first_seen else oracle.ORDER_ASCENDING
    seen = np.zeros(n_nodes, dtype=bool)
    start = 0
    for seg in range(2):
        sizes = [min(n_nodes, x) for x in ([40, 0, 17, 64, 5, 1, 33, 80, 2, 9, 50, 12, 7, 3, 21, 60][:group])]
        seeds_np = [rng.choice(n_nodes, size=k, replace=False).astype(np.int32) for k in sizes]
        outs = [B.BlockBuffers(n_nodes, ci.size, max(k, 1), fanouts, DEV) for k in sizes]
        ctx.sample_blocks_group(csr, [_i32(x) if x.size else torch.empty(0, dtype=torch.int32, device=DEV) for x in seeds_np],
                                fanouts, 11, seg, outs, node_order=B.RG_ORDER_FIRST_SEEN if first_seen else B.RG_ORDER_ASCENDING)
        ctx.plan_sampled(group, cache, claimed, plan, seg)
        torch.cuda.synchronize()
        new = np.zeros(n_nodes, dtype=bool)
        for x in seeds_np:
            new[oracle.sample_blocks(rp, ci, x, fanouts, 11, seg, order).input_nodes] = True
        new &= ~seen
        seen |= new
        rows = home_np[np.flatnonzero(new & remote)] & 0x3FFFFFFF
        offs = plan.offsets.cpu().numpy()
        assert offs[seg] == start and offs[seg + 1] == start + rows.size, (seg, offs[:3], rows.size)
        pairs = plan.list.cpu().numpy()[2 * start:2 * (start + rows.size)].reshape(-1, 2)
        assert np.array_equal(pairs[:, 0], rows) and np.array_equal(pairs[:, 1], rows)
        cl = np.unpackbits(claimed.cpu().numpy().view(np.uint8), bitorder="little")
        assert np.array_equal(cl[:n_nodes].astype(bool), seen) and not cl[n_nodes:].any()
        start += rows.size


@pytest.mark.parametrize("histogram,node_order", [("epoch", "ascending"), ("sampled", "ascending"), ("sampled", "first_seen"),
                                                  ("batch", "first_seen")])
@pytest.mark.parametrize("full_cache", [False, True])
@pytest.mark.parametrize("double_buffer", [False, True])
def test_pipeline_epochs_back_to_back(B, double_buffer, full_cache, histogram, node_order):
    """Three epochs through EpochPipeline.run_epochs; with double buffering epoch e+1 is precomputed and its rows
    pulled while epoch e is served.  Every batch's rows and statistics and every epoch's cache are checked, with the
    access counts taken by the epoch pass over the id lists, straight from the sampler's bitmaps, or batch by batch,
    and with either node order."""
    log(f"[pipeline epochs] double_buffer={double_buffer} full_cache={full_cache} histogram={histogram} node_order={node_order}")
    order = oracle.ORDER_FIRST_SEEN if node_order == "first_seen" else oracle.ORDER_ASCENDING
    import dataclasses
    from paper_2505_10806_amd.pipeline import EpochPipeline
    base = synth.get_config("tiny")
    # full_cache: the cache can hold every remote node, so every touched remote row is selected and no row misses
    wl = synth.build_workload(dataclasses.replace(base, cache_frac=1.0) if full_cache else base, seed=5, device=DEV)
    cfg = wl.cfg
    rp, ci = host_graph(wl)
    X = wl.features.cpu().numpy()
    home_np, train_np = wl.home.cpu().numpy(), wl.train_ids.cpu().numpy()
    # a mirrored cache is filled by one pull per sampler call (lists off the bitmaps) or one per batch: cover both
    pulls = "batch" if (full_cache and histogram == "epoch") else "group"
    pipe = EpochPipeline(wl, device=DEV, double_buffer=double_buffer, histogram=histogram, node_order=node_order, mirror_pulls=pulls)
    nb = pipe.batches_per_epoch
    expected = {}

    def epoch_start(p, k):                      # oracle results for the epoch that is about to be served
        torch.cuda.synchronize()                # its offline stage runs on streams of its own
        batches = oracle.epoch_batches(train_np, cfg.batch_size, wl.seed, k, cfg.max_batches)
        counts = np.zeros(cfg.num_nodes, dtype=np.uint32)
        inputs = []
        for seeds in batches:
            blk = oracle.sample_blocks(rp, ci, seeds, cfg.fanouts, wl.seed, k, order)
            oracle.access_histogram(blk.input_nodes, counts)
            inputs.append(blk.input_nodes)
        ids, loc = oracle.build_cache(counts, home_np, wl.capacity_rows)
        expected[k] = (inputs, counts, ids, loc)
        for b, nodes in enumerate(inputs):
            assert np.array_equal(p.arena[b, :nodes.size].cpu().numpy(), nodes), f"input nodes of epoch {k} batch {b}"
        assert np.array_equal(p.counts.cpu().numpy().view(np.uint32), counts)
        assert np.array_equal(p.cache.cache_ids[:ids.size].cpu().numpy(), ids)
        assert np.array_equal(p.cache.loc.cpu().numpy(), loc)
        p._epoch = k

    def batch_done(p, b):
        torch.cuda.synchronize()
        inputs, _, _, loc = expected[p._epoch]
        want, st = oracle.gather_features(X, inputs[b], loc)
        n = inputs[b].size
        assert p.sizes[b] == n
        assert np.array_equal(p.out[:n, :cfg.feat_dim].cpu().numpy(), want), f"epoch {p._epoch} batch {b}"
        assert tuple(p.stats[b].cpu().tolist()) == st

    def epoch_done(p, k):
        torch.cuda.synchronize()
        _, _, ids, _ = expected[k]
        rows = p.cache.rows_of(torch.as_tensor(ids, device=DEV))      # slots, or remote-store rows for a mirrored cache
        assert p.mirror == full_cache
        if not p.mirror:
            assert np.array_equal(rows.cpu().numpy(), np.arange(ids.size))
        assert np.array_equal(p.cache.cache_rows[rows, :cfg.feat_dim].cpu().numpy(), X[ids])

    pipe.run_epochs(0, 3, nb, on_epoch_done=epoch_done, on_batch=batch_done, on_epoch_start=epoch_start)
    torch.cuda.synchronize()
    assert sorted(expected) == [0, 1, 2]
    assert not np.array_equal(expected[0][0][0], expected[1][0][0])       # epochs differ


def _oracle_period(wl, rp, ci, home_np, train_np, first_epoch, epochs):
    """Oracle input nodes of every batch of the listed epochs, and the counts over all of them."""
    cfg = wl.cfg
    counts = np.zeros(cfg.num_nodes, dtype=np.uint32)
    inputs = []
    for e in range(first_epoch, first_epoch + epochs):
        for seeds in oracle.epoch_batches(train_np, cfg.batch_size, wl.seed, e, cfg.max_batches):
            blk = oracle.sample_blocks(rp, ci, seeds, cfg.fanouts, wl.seed, e)
            oracle.access_histogram(blk.input_nodes, counts)
            inputs.append(blk.input_nodes)
    return inputs, counts


@pytest.mark.parametrize("mirror_pulls", ["group", "batch"])
@pytest.mark.parametrize("double_buffer", [False, True])
def test_pipeline_keeps_rows_of_earlier_epochs(B, double_buffer, mirror_pulls):
    """keep_rows on a cache that mirrors the remote store: features do not change, so an epoch pulls only the rows that
    no earlier epoch has named.  Three epochs; every batch's rows and statistics and each epoch's TopHot result against
    the oracle (which knows nothing of kept rows: the result must not depend on them); after each epoch the resident
    rows are exactly the remote nodes named so far, each holding its feature row, and nothing else was written."""
    import dataclasses
    from paper_2505_10806_amd.pipeline import EpochPipeline
    wl = synth.build_workload(dataclasses.replace(synth.CONFIGS["tiny"], cache_frac=1.0), seed=12, device=DEV)
    cfg = wl.cfg
    rp, ci = host_graph(wl)
    X = wl.features.cpu().numpy()
    home_np, train_np = wl.home.cpu().numpy(), wl.train_ids.cpu().numpy()
    tag = (home_np.astype(np.int64) & 0xFFFFFFFF) >> 30
    remote_ids = np.flatnonzero(tag == 2)
    assert np.array_equal(home_np[remote_ids].astype(np.int64) & 0x3FFFFFFF, np.arange(remote_ids.size))   # row = rank among the remote ids
    pipe = EpochPipeline(wl, device=DEV, double_buffer=double_buffer, keep_rows=True, mirror_pulls=mirror_pulls)
    assert pipe.mirror and pipe.keep_rows
    pipe.cache.cache_rows.fill_(float("nan"))
    nb = pipe.batches_per_epoch
    expected, named, resident_counts = {}, np.zeros(cfg.num_nodes, dtype=bool), []

    def epoch_start(p, k):
        torch.cuda.synchronize()
        inputs, counts = _oracle_period(wl, rp, ci, home_np, train_np, k, 1)
        ids, loc = oracle.build_cache(counts, home_np, wl.capacity_rows)
        expected[k] = (inputs, loc)
        assert np.array_equal(p.cache.cache_ids[:ids.size].cpu().numpy(), ids) and int(p.cache.num_cached.item()) == ids.size
        assert np.array_equal(p.cache.loc.cpu().numpy(), loc)
        p._epoch = k

    def batch_done(p, b):
        torch.cuda.synchronize()
        inputs, loc = expected[p._epoch]
        want, st = oracle.gather_features(X, inputs[b], loc)
        assert st[2] == 0 and tuple(p.stats[b].cpu().tolist()) == st
        assert np.array_equal(p.out[:inputs[b].size, :cfg.feat_dim].cpu().numpy(), want), f"epoch {p._epoch} batch {b}"

    def epoch_done(p, k):
        torch.cuda.synchronize()
        for nodes in expected[k][0]:
            named[nodes] = True
        bits = np.unpackbits(p.cache.filled.cpu().numpy().view(np.uint8), bitorder="little")[:wl.n_remote].astype(bool)
        if not double_buffer:                     # (with the double buffer the next epoch's pulls are already under way)
            assert np.array_equal(bits, named[remote_ids])
            got = p.cache.cache_rows.cpu().numpy()
            assert np.array_equal(got[bits, :cfg.feat_dim], X[remote_ids[bits]]) and np.isnan(got[~bits]).all()
        else:
            assert bits[named[remote_ids]].all()
        resident_counts.append(int(named[remote_ids].sum()))

    pipe.run_epochs(0, 3, nb, on_epoch_done=epoch_done, on_batch=batch_done, on_epoch_start=epoch_start)
    torch.cuda.synchronize()
    bits = np.unpackbits(pipe.cache.filled.cpu().numpy().view(np.uint8), bitorder="little")[:wl.n_remote].astype(bool)
    assert np.array_equal(bits, named[remote_ids])
    got = pipe.cache.cache_rows.cpu().numpy()
    assert np.array_equal(got[bits, :cfg.feat_dim], X[remote_ids[bits]]) and np.isnan(got[~bits]).all()
    assert resident_counts[0] < resident_counts[1] < resident_counts[2] < wl.n_remote     # each epoch added rows, none named them all
    pipe.close()


@pytest.mark.parametrize("full_cache", [False, True])
def test_pipeline_with_compute_units_split_between_pulls_and_the_rest(B, full_cache):
    """pull_cus: the prefetch stream is bound to a few compute units, every other stream of the pipeline (and the
    stream the gathers run on) to the rest.  Placement changes nothing in the results: two epochs, double buffered,
    every batch's rows and statistics and each epoch's cache against the oracle."""
    import dataclasses
    from paper_2505_10806_amd.pipeline import EpochPipeline
    base = synth.CONFIGS["tiny"]
    wl = synth.build_workload(dataclasses.replace(base, cache_frac=1.0) if full_cache else base, seed=9, device=DEV)
    cfg = wl.cfg
    rp, ci = host_graph(wl)
    X = wl.features.cpu().numpy()
    home_np, train_np = wl.home.cpu().numpy(), wl.train_ids.cpu().numpy()
    pipe = EpochPipeline(wl, device=DEV, double_buffer=True, pull_cus=16)
    assert pipe.work_stream is not None and pipe.mirror == full_cache
    nb = pipe.batches_per_epoch
    expected, seen = {}, []

    def epoch_start(p, k):
        torch.cuda.synchronize()
        inputs, counts = _oracle_period(wl, rp, ci, home_np, train_np, k, 1)
        ids, loc = oracle.build_cache(counts, home_np, wl.capacity_rows)
        expected[k] = (inputs, loc)
        assert np.array_equal(p.counts.cpu().numpy().view(np.uint32), counts)
        assert np.array_equal(p.cache.cache_ids[:ids.size].cpu().numpy(), ids)
        assert np.array_equal(p.cache.loc.cpu().numpy(), loc)
        p._epoch = k

    def batch_done(p, b):
        torch.cuda.synchronize()
        inputs, loc = expected[p._epoch]
        want, st = oracle.gather_features(X, inputs[b], loc)
        assert np.array_equal(p.out[:inputs[b].size, :cfg.feat_dim].cpu().numpy(), want), f"epoch {p._epoch} batch {b}"
        assert tuple(p.stats[b].cpu().tolist()) == st
        seen.append((p._epoch, b))

    with torch.cuda.stream(pipe.work_stream):
        pipe.run_epochs(0, 2, nb, on_batch=batch_done, on_epoch_start=epoch_start)
    torch.cuda.synchronize()
    assert seen == [(k, b) for k in (0, 1) for b in range(nb)]
    pipe.close()


def test_streams_on_a_share_of_the_compute_units(B):
    """rg_stream_create / rg_stream_destroy: a gather on a stream bound to 8 compute units gives the oracle's rows; ranges
    outside the device and foreign streams are refused."""
    c = B.Context(0)
    n_cus = c.num_cus
    s = c.stream_on_cus(n_cus - 8, 8)
    wl = synth.build_workload("tiny", seed=4, device=DEV)
    cfg = wl.cfg
    X = wl.features.cpu().numpy()
    home_np = wl.home.cpu().numpy()
    g = torch.Generator().manual_seed(1)
    nodes = torch.randint(0, cfg.num_nodes, (5000,), generator=g, dtype=torch.int32)
    counts_orc = np.zeros(cfg.num_nodes, dtype=np.uint32)
    oracle.access_histogram(nodes.numpy(), counts_orc)
    ids_orc, loc_orc = oracle.build_cache(counts_orc, home_np, wl.capacity_rows)
    nodes_dev = nodes.to(DEV)
    counts = torch.zeros(cfg.num_nodes, dtype=torch.int32, device=DEV)
    cache = B.FeatureCache(cfg.num_nodes, wl.capacity_rows, wl.stride, DEV)
    out = torch.zeros(nodes.numel(), wl.stride, device=DEV)
    stats = torch.zeros(3, dtype=torch.int64, device=DEV)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        c.access_histogram(nodes_dev, nodes.numel(), counts)
        c.build_cache(counts, wl.home, wl.remote_store, cfg.feat_dim, cache)
        c.gather_features(nodes_dev, nodes.numel(), cache, wl.local_store, wl.remote_store, cfg.feat_dim, out, stats)
    s.synchronize()
    want, st = oracle.gather_features(X, nodes.numpy(), loc_orc)
    assert tuple(stats.cpu().tolist()) == st and st[1] > 0 and st[2] > 0
    assert np.array_equal(out[:, :cfg.feat_dim].cpu().numpy(), want)
    for first, n in ((0, 0), (-1, 4), (n_cus - 3, 4), (0, n_cus + 1)):
        with pytest.raises(B.RgError):
            c.stream_on_cus(first, n)
    assert B._lib.rg_stream_destroy(c._h, 0x1234) != B.RG_OK           # not one of this context's streams
    assert B._lib.rg_stream_destroy(c._h, s.cuda_stream) == B.RG_OK
    assert B._lib.rg_stream_destroy(c._h, s.cuda_stream) != B.RG_OK           # already gone
    c.close()


@pytest.mark.parametrize("full_cache", [False, True])
@pytest.mark.parametrize("double_buffer", [False, True])
def test_pipeline_period_of_two_epochs_shares_one_cache(B, double_buffer, full_cache):
    """Alg. 1 lines 1-4 as written: the batches of all precomputed epochs are counted together and one steady cache
    serves them.  Two periods of two epochs each; every slot's input nodes, the period's counts, cache and location
    table, and every batch's rows and statistics against the oracle; then the comparison with a cache per epoch:
    the per-epoch caches serve at least as many requests, the shared cache is filled once instead of twice."""
    import dataclasses
    from paper_2505_10806_amd.pipeline import EpochPipeline
    # full_cache: the cache mirrors the remote store and is filled by one pull per sampler call, across both epochs of a period
    base = synth.CONFIGS["tiny"]
    wl = synth.build_workload(dataclasses.replace(base, cache_frac=1.0) if full_cache else base, seed=5, device=DEV)
    cfg = wl.cfg
    rp, ci = host_graph(wl)
    X = wl.features.cpu().numpy()
    home_np, train_np = wl.home.cpu().numpy(), wl.train_ids.cpu().numpy()
    pipe = EpochPipeline(wl, device=DEV, double_buffer=double_buffer, period_epochs=2)
    assert pipe.mirror == full_cache
    nb = pipe.batches_per_epoch
    expected, hits = {}, {}

    def period_start(p, k):
        torch.cuda.synchronize()                # the period's offline stage runs on streams of its own
        inputs, counts = _oracle_period(wl, rp, ci, home_np, train_np, 2 * k, 2)
        ids, loc = oracle.build_cache(counts, home_np, wl.capacity_rows)
        expected[k] = (inputs, counts, ids, loc)
        assert p.n_batches == 2 * nb == len(inputs)
        for i, nodes in enumerate(inputs):
            assert np.array_equal(p.arena[i, :nodes.size].cpu().numpy(), nodes), f"period {k} slot {i}"
        assert np.array_equal(p.counts.cpu().numpy().view(np.uint32), counts)
        assert np.array_equal(p.cache.cache_ids[:ids.size].cpu().numpy(), ids)
        assert np.array_equal(p.cache.loc.cpu().numpy(), loc)
        p._period = k
        hits[k] = [0, 0]

    def batch_done(p, i):
        torch.cuda.synchronize()
        inputs, _, _, loc = expected[p._period]
        want, st = oracle.gather_features(X, inputs[i], loc)
        assert np.array_equal(p.out[:inputs[i].size, :cfg.feat_dim].cpu().numpy(), want), f"period {p._period} slot {i}"
        assert tuple(p.stats[i].cpu().tolist()) == st
        hits[p._period][0] += st[1]
        hits[p._period][1] += st[2]

    pipe.run_epochs(0, 2, nb, on_batch=batch_done, on_epoch_start=period_start)
    torch.cuda.synchronize()
    remote = ((home_np.astype(np.int64) & 0xFFFFFFFF) >> 30) == 2
    for k in (0, 1):
        _, counts, ids, _ = expected[k]
        assert hits[k][0] == int(counts[ids].sum()) and sum(hits[k]) == int(counts[remote].sum())   # closed form
    # the same two epochs with a cache per epoch (oracle): at least as many hits, twice the fill
    per_epoch_hits = per_epoch_fill = 0
    for e in (0, 1):
        _, c_e = _oracle_period(wl, rp, ci, home_np, train_np, e, 1)
        ids_e, _ = oracle.build_cache(c_e, home_np, wl.capacity_rows)
        per_epoch_hits += int(c_e[ids_e].sum())
        per_epoch_fill += ids_e.size
    assert per_epoch_hits >= hits[0][0]
    if full_cache:        # every named remote row is cached either way; the shared cache pulls the rows both epochs name once
        assert per_epoch_hits == hits[0][0] and expected[0][2].size < per_epoch_fill < 2 * expected[0][2].size
    else:
        assert per_epoch_fill == 2 * expected[0][2].size


def test_group_partition_cuts_remote_requests(B):
    """The `small` shapes on a graph with four planted groups, partitioned at random and along the groups (the stand-in
    for an edge-cut-minimising partitioner), seeds from the local partition: the whole path against the oracle on
    three batches of each, then the comparison the paper draws between its partitioners: far fewer requests for
    remote rows, and fewer remote fetches after the cache, along the groups."""
    from paper_2505_10806_amd.pipeline import EpochPipeline
    remote_requests, misses = {}, {}
    for name in ("small_groups_random", "small_groups_local"):
        wl = synth.build_workload(name, seed=2025, device=DEV)
        cfg = wl.cfg
        rp, ci = host_graph(wl)
        X = wl.features.cpu().numpy()
        home_np, train_np = wl.home.cpu().numpy(), wl.train_ids.cpu().numpy()
        pipe = EpochPipeline(wl, device=DEV)
        nb = pipe.batches_per_epoch
        pipe.run_epoch(0, nb)
        torch.cuda.synchronize()
        stats = pipe.stats[:nb].cpu().numpy()
        counts = pipe.counts.cpu().numpy().view(np.uint32)
        remote = ((home_np.astype(np.int64) & 0xFFFFFFFF) >> 30) == 2
        k = int(pipe.cache.num_cached.item())
        ids = pipe.cache.cache_ids[:k].cpu().numpy()
        assert stats[:, 1].sum() == int(counts[ids].sum()) and stats[:, 1:].sum() == int(counts[remote].sum())
        batches = oracle.epoch_batches(train_np, cfg.batch_size, wl.seed, 0)
        assert len(batches) == nb
        counts_orc = np.zeros(cfg.num_nodes, dtype=np.uint32)
        inputs = []
        for seeds in batches:
            blk = oracle.sample_blocks(rp, ci, seeds, cfg.fanouts, wl.seed, 0)
            oracle.access_histogram(blk.input_nodes, counts_orc)
            inputs.append(blk.input_nodes)
        assert np.array_equal(counts, counts_orc)
        ids_orc, loc_orc = oracle.build_cache(counts_orc, home_np, wl.capacity_rows)
        assert np.array_equal(ids, ids_orc) and np.array_equal(pipe.cache.loc.cpu().numpy(), loc_orc)
        for b in (0, nb // 2, nb - 1):
            assert np.array_equal(pipe.arena[b, :inputs[b].size].cpu().numpy(), inputs[b])
            _, st = oracle.gather_features(X[:, :1], inputs[b], loc_orc)
            assert tuple(stats[b].tolist()) == st
        want, _ = oracle.gather_features(X, inputs[nb - 1], loc_orc)          # the last gather's rows are still in pipe.out
        assert np.array_equal(pipe.out[:inputs[nb - 1].size, :cfg.feat_dim].cpu().numpy(), want)
        remote_requests[name] = int(stats[:, 1:].sum())
        misses[name] = int(stats[:, 2].sum())
        log(f"[partition] {name}: rows {int(stats.sum())}, requests for remote rows {remote_requests[name]}, "
            f"hits {int(stats[:, 1].sum())}, remote fetches {misses[name]}, cached rows {k}")
    assert remote_requests["small_groups_local"] < 0.5 * remote_requests["small_groups_random"]
    assert misses["small_groups_local"] < misses["small_groups_random"]


@pytest.mark.parametrize("num_batches", [0, 1, 7, 1023, 1500])
def test_prefetch_plan_groups_slots_by_first_batch(B, ctx, num_batches):
    """rg_plan_prefetch on a synthetic first-use array: segment b holds exactly the slots whose node is first
    needed by batch b (ascending for up to 1023 batches), segment num_batches the slots no batch uses."""
    log(f"[prefetch plan] num_batches={num_batches}")
    rng = np.random.default_rng(num_batches)
    n, dim = 20_000, 8
    is_local = torch.from_numpy(rng.random(n) < 0.3)
    home = synth.stores.make_home(is_local)
    home_np = home.numpy()
    counts = rng.integers(0, 3, size=n).astype(np.uint32)
    first = rng.integers(0, max(num_batches, 1) + 3, size=n).astype(np.uint32)      # some beyond the planned batches
    first[rng.integers(0, n, 50)] = 0xFFFFFFFF
    cache = B.FeatureCache(n, 6000, dim, DEV)
    ctx.build_cache(torch.from_numpy(counts.view(np.int32)).to(DEV), home.to(DEV), None, dim, cache)
    plan = B.PrefetchPlan(6000, num_batches, DEV)
    ctx.plan_prefetch(cache, home.to(DEV), torch.from_numpy(first.view(np.int32)).to(DEV), plan)
    torch.cuda.synchronize()
    ids_orc, _ = oracle.build_cache(counts, home_np, 6000)
    k = ids_orc.size
    key = np.minimum(first[ids_orc].astype(np.int64), num_batches)
    offs = plan.offsets.cpu().numpy()
    pairs = plan.list.cpu().numpy().reshape(-1, 2)
    assert offs[0] == 0 and offs[num_batches + 1] == k
    for b in range(num_batches + 1):
        seg = pairs[offs[b]:offs[b + 1]]
        want_slots = np.flatnonzero(key == b)
        if num_batches + 1 <= 1024:
            assert np.array_equal(seg[:, 0], want_slots), b
        else:
            assert np.array_equal(np.sort(seg[:, 0]), want_slots), b
        assert np.array_equal(seg[:, 1], (home_np[ids_orc[seg[:, 0]]].astype(np.int64) & 0x3FFFFFFF)), b


# ------------------------------------------------------------------------------ TopHot edge cases
@pytest.mark.parametrize("capacity", [0, 1, 5, 1000, 4000, 1 << 20])
def test_build_cache_edge_cases(B, ctx, capacity):
    log(f"[build_cache] capacity={capacity}")
    rng = np.random.default_rng(capacity + 1)
    n, dim = 5000, 12
    is_local = torch.from_numpy(rng.random(n) < 0.25)
    home = synth.stores.make_home(is_local)
    counts = rng.integers(0, 4, size=n).astype(np.uint32)                 # heavy ties and zeros
    counts[rng.integers(0, n, 6)] = np.uint32(2 ** 31 + 7)                # counts beyond int32
    counts[rng.integers(0, n, 3)] = np.uint32(2 ** 32 - 1)
    X = rng.standard_normal((n, dim)).astype(np.float32)
    stride = synth.stores.row_stride(dim)
    remote = torch.zeros(int((~is_local).sum()), stride, pin_memory=True)
    remote[:, :dim] = torch.from_numpy(X)[~is_local]
    cache = B.FeatureCache(n, min(capacity, n), stride, DEV)
    cache.c_struct.capacity_rows = capacity          # the buffers hold min(capacity, n) rows, which bounds K_eff
    ctx.build_cache(torch.from_numpy(counts.view(np.int32)).to(DEV), home.to(DEV), remote, dim, cache)
    torch.cuda.synchronize()
    ids_orc, loc_orc = oracle.build_cache(counts, home.numpy(), min(capacity, n))
    k = int(cache.num_cached.item())
    assert k == ids_orc.size
    assert np.array_equal(cache.cache_ids[:k].cpu().numpy(), ids_orc)
    assert np.array_equal(cache.loc.cpu().numpy(), loc_orc)
    assert np.array_equal(cache.cache_rows[:k, :dim].cpu().numpy(), X[ids_orc])


def test_build_cache_on_generated_counts(B, ctx):
    """Randomised TopHot: counts with heavy ties, zeros and values on every byte boundary of the radix select."""
    from hypothesis import HealthCheck, given, settings, strategies as st
    special = [0, 1, 2, 255, 256, 257, 65535, 65536, 2 ** 24 - 1, 2 ** 24, 2 ** 31, 2 ** 32 - 1]

    @st.composite
    def case(draw):
        n = draw(st.integers(1, 2500))
        pool = draw(st.lists(st.sampled_from(special) | st.integers(0, 5), min_size=1, max_size=6))
        seed = draw(st.integers(0, 2 ** 31))
        cap = draw(st.sampled_from([0, 1, 2, 7, 64, 500, 2499, 2500, 10 ** 6]))
        p_local = draw(st.sampled_from([0.0, 0.3, 1.0]))
        return n, pool, seed, cap, p_local

    @settings(max_examples=80, deadline=None, derandomize=True, suppress_health_check=list(HealthCheck))
    @given(case())
    def run(c):
        n, pool, seed, cap, p_local = c
        rng = np.random.default_rng(seed)
        counts = np.array(pool, dtype=np.uint64)[rng.integers(0, len(pool), size=n)].astype(np.uint32)
        home = synth.stores.make_home(torch.from_numpy(rng.random(n) < p_local))
        cache = B.FeatureCache(n, min(cap, n), 4, DEV)
        cache.c_struct.capacity_rows = cap
        ctx.build_cache(torch.from_numpy(counts.view(np.int32)).to(DEV), home.to(DEV), None, 4, cache)
        torch.cuda.synchronize()
        ids_orc, loc_orc = oracle.build_cache(counts, home.numpy(), cap)
        k = int(cache.num_cached.item())
        assert k == ids_orc.size
        assert np.array_equal(cache.cache_ids[:k].cpu().numpy(), ids_orc)
        assert np.array_equal(cache.loc.cpu().numpy(), loc_orc)
        hits, total = ctx.cache_hit_curve(torch.from_numpy(counts.view(np.int32)).to(DEV), home.to(DEV), [cap])
        torch.cuda.synchronize()
        want_hits, want_total = oracle.cache_hit_curve(counts, home.numpy(), [cap])
        assert int(hits[0].item()) == int(want_hits[0]) and int(total.item()) == want_total

    run()


def test_build_cache_all_local(B, ctx):
    n = 300
    home = synth.stores.make_home(torch.ones(n, dtype=torch.bool))
    counts = torch.ones(n, dtype=torch.int32, device=DEV)
    remote = torch.zeros(1, 4, pin_memory=True)
    cache = B.FeatureCache(n, 10, 4, DEV)
    ctx.build_cache(counts, home.to(DEV), remote, 4, cache)
    torch.cuda.synchronize()
    assert int(cache.num_cached.item()) == 0
    assert np.array_equal(cache.loc.cpu().numpy(), home.numpy())


def test_cache_hit_curve(B, ctx):
    rng = np.random.default_rng(77)
    n = 40_000
    home = synth.stores.make_home(torch.from_numpy(rng.random(n) < 0.25))
    counts = (rng.zipf(1.6, size=n) % 300).astype(np.uint32)
    counts[rng.integers(0, n, 4)] = np.uint32(2 ** 31 + 11)
    counts[rng.integers(0, n, 2000)] = 0
    caps = [0, 1, 2, 17, 1000, 5000, 20_000, 29_999, 30_000, 10 ** 6]
    hits, total = ctx.cache_hit_curve(torch.from_numpy(counts.view(np.int32)).to(DEV), home.to(DEV), caps)
    torch.cuda.synchronize()
    want, want_total = oracle.cache_hit_curve(counts, home.numpy(), caps)
    assert hits.cpu().numpy().astype(np.uint64).tolist() == want.tolist()
    assert int(total.item()) == want_total
    # no capacities: only the total; no remote nodes: everything zero
    hits, total = ctx.cache_hit_curve(torch.from_numpy(counts.view(np.int32)).to(DEV), home.to(DEV), [])
    torch.cuda.synchronize()
    assert hits.numel() == 0 and int(total.item()) == want_total
    all_local = synth.stores.make_home(torch.ones(n, dtype=torch.bool))
    hits, total = ctx.cache_hit_curve(torch.from_numpy(counts.view(np.int32)).to(DEV), all_local.to(DEV), [5, 50])
    torch.cuda.synchronize()
    assert hits.cpu().tolist() == [0, 0] and int(total.item()) == 0


def test_batch_salted_seed_gives_per_batch_streams(B, ctx):
    """The draw is keyed by (seed, epoch, node, hop).  A caller that wants the streams to differ between batches
    as well (the paper's "epochs and batches") folds the batch index into the 64-bit seed; the oracle then
    reproduces each batch with the same folded seed."""
    rng = np.random.default_rng(5)
    rp, ci = _handmade_graph(400, 0.6, 30, 0.02, rng)
    csr = B.CsrGraph(torch.as_tensor(rp, device=DEV), _i32(ci))
    seeds = np.arange(0, 30, dtype=np.int32)                 # the dense core: degrees above the fan-out
    rows = []
    for batch in range(3):
        salted = (2025 + (batch << 32)) & (2 ** 64 - 1)
        hip = _run_blocks(B, ctx, csr, seeds, (5, 3), salted, 1)
        orc = oracle.sample_blocks(rp, ci, seeds, (5, 3), salted, 1)
        assert_batch_equal(hip, orc, 2, f"batch {batch}")
        rows.append(hip.nbr[0].tolist())
    assert rows[0] != rows[1] and rows[1] != rows[2]
    again = _run_blocks(B, ctx, csr, seeds, (5, 3), 2025, 1)
    assert again.nbr[0].tolist() == rows[0]                   # batch 0's salt is zero


# ------------------------------------------------------------------------------ gather shapes
@pytest.mark.parametrize("dim,pad", [(64, True), (100, True), (128, True), (256, True), (602, True), (602, False),
                                     (7, False), (7, True), (257, False), (1, False), (1000, True)])
@pytest.mark.parametrize("two_streams", [False, True])
def test_gather_shapes_and_tags(B, ctx, dim, pad, two_streams):
    log(f"[gather] dim={dim} pad={pad} two_streams={two_streams}")
    rng = np.random.default_rng(dim * 2 + pad)
    n_nodes, n_local, n_cache, n_remote = 3000, 900, 500, 2100
    stride = synth.stores.row_stride(dim) if pad else dim
    X = rng.standard_normal((n_nodes, dim)).astype(np.float32)
    perm = rng.permutation(n_nodes)
    loc = np.zeros(n_nodes, dtype=np.int64)
    local_ids, remote_ids = perm[:n_local], perm[n_local:]
    cached_ids = remote_ids[:n_cache]
    loc[local_ids] = (0 << 30) | np.arange(n_local)
    loc[remote_ids] = (2 << 30) | np.arange(n_remote)
    loc[cached_ids] = (1 << 30) | np.arange(n_cache)
    loc32 = loc.astype(np.uint32).view(np.int32)

    def pack(ids, pinned):
        t = torch.zeros(len(ids), stride, pin_memory=True) if pinned else torch.zeros(len(ids), stride)
        t[:, :dim] = torch.from_numpy(X[ids])
        return t if pinned else t.to(DEV)
    local_store, remote_store = pack(local_ids, False), pack(remote_ids, True)
    cache = B.FeatureCache(n_nodes, n_cache, stride, DEV)
    cache.cache_rows[:, :dim] = torch.from_numpy(X[cached_ids]).to(DEV)
    cache.loc.copy_(torch.from_numpy(loc32))
    stats = torch.zeros(3, dtype=torch.int64, device=DEV)
    side = torch.cuda.Stream() if two_streams else None
    for n in (0, 1, 63, 257, 4097):
        nodes = rng.integers(0, n_nodes, size=n).astype(np.int32)         # repeats allowed
        out = torch.full((max(n, 1), stride), float("nan"), device=DEV)
        nodes_dev = torch.as_tensor(nodes, device=DEV) if n else torch.empty(1, dtype=torch.int32, device=DEV)
        ctx.gather_features(nodes_dev, n, cache, local_store, remote_store, dim, out, stats, miss_stream=side)
        torch.cuda.synchronize()
        want, st = oracle.gather_features(X, nodes, loc32)
        assert np.array_equal(out[:n, :dim].cpu().numpy(), want), f"n={n}"
        assert tuple(stats.cpu().tolist()) == st
        assert torch.isnan(out[:, dim:]).all(), "the padding behind an output row was written"
    # count read from the device: the launch is sized for 4097 rows but only 1000 are valid
    nodes = rng.integers(0, n_nodes, size=4097).astype(np.int32)
    n_dev = torch.tensor([1000], dtype=torch.int32, device=DEV)
    out = torch.full((4097, stride), float("nan"), device=DEV)
    ctx.gather_features(torch.as_tensor(nodes, device=DEV), 4097, cache, local_store, remote_store, dim, out, stats,
                        n_dev=n_dev, miss_stream=side)
    torch.cuda.synchronize()
    want, st = oracle.gather_features(X, nodes[:1000], loc32)
    assert np.array_equal(out[:1000, :dim].cpu().numpy(), want)
    assert torch.isnan(out[1000:, :dim]).all()
    assert tuple(stats.cpu().tolist()) == st


def test_gather_with_stale_cache_and_misaligned_buffers(B, ctx):
    """A cache selected for another epoch changes the hit rate, never the rows; buffers that are only 4-byte aligned
    fall back to scalar accesses and still copy exactly dim floats."""
    wl = synth.build_workload("tiny", seed=41, device=DEV)
    cfg = wl.cfg
    H = len(cfg.fanouts)
    rp, ci = host_graph(wl)
    X = wl.features.cpu().numpy()
    home_np, train_np = wl.home.cpu().numpy(), wl.train_ids.cpu().numpy()
    counts0 = np.zeros(cfg.num_nodes, dtype=np.uint32)
    for seeds in oracle.epoch_batches(train_np, cfg.batch_size, wl.seed, 0, 4):
        oracle.access_histogram(oracle.sample_blocks(rp, ci, seeds, cfg.fanouts, wl.seed, 0).input_nodes, counts0)
    cache = B.FeatureCache(cfg.num_nodes, wl.capacity_rows, wl.stride, DEV)
    ctx.build_cache(torch.from_numpy(counts0.view(np.int32)).to(DEV), wl.home, wl.remote_store, cfg.feat_dim, cache)
    _, loc0 = oracle.build_cache(counts0, home_np, wl.capacity_rows)
    seeds1 = oracle.epoch_batches(train_np, cfg.batch_size, wl.seed, 1, 4)[2]          # a batch of the next epoch
    blk = oracle.sample_blocks(rp, ci, seeds1, cfg.fanouts, wl.seed, 1)
    nodes = torch.as_tensor(blk.input_nodes, device=DEV)
    n = blk.input_nodes.size
    stats = torch.zeros(3, dtype=torch.int64, device=DEV)
    want, st = oracle.gather_features(X, blk.input_nodes, loc0)
    # aligned, padded output
    out = torch.full((n, wl.stride), float("nan"), device=DEV)
    ctx.gather_features(nodes, n, cache, wl.local_store, wl.remote_store, cfg.feat_dim, out, stats)
    torch.cuda.synchronize()
    assert np.array_equal(out[:, :cfg.feat_dim].cpu().numpy(), want) and tuple(stats.cpu().tolist()) == st
    assert 0 < st[1] and 0 < st[2]                                                    # still some hits, more misses
    # output that starts 4 bytes into an allocation, row stride = dim + 1: scalar path, neighbours untouched
    flat = torch.full((n * (cfg.feat_dim + 1) + 1,), float("nan"), device=DEV)
    out2 = flat[1:].view(n, cfg.feat_dim + 1)
    assert out2.data_ptr() % 16 == 4
    ctx.gather_features(nodes, n, cache, wl.local_store, wl.remote_store, cfg.feat_dim, out2, stats)
    torch.cuda.synchronize()
    assert np.array_equal(out2[:, :cfg.feat_dim].cpu().numpy(), want)
    assert torch.isnan(out2[:, cfg.feat_dim]).all() and torch.isnan(flat[0])
    assert tuple(stats.cpu().tolist()) == st


def test_gather_prepare_group_then_run(B, ctx):
    """Several batches classified by one launch, copied later ticket by ticket in any order, on another stream;
    a ticket that was not prepared for the same row count is refused."""
    rng = np.random.default_rng(12)
    n_nodes, dim = 4000, 20
    stride = synth.stores.row_stride(dim)
    X = rng.standard_normal((n_nodes, dim)).astype(np.float32)
    is_local = torch.from_numpy(rng.random(n_nodes) < 0.4)
    home = synth.stores.make_home(is_local)
    local = torch.zeros(int(is_local.sum()), stride, device=DEV)
    local[:, :dim] = torch.from_numpy(X)[is_local].to(DEV)
    remote = torch.zeros(int((~is_local).sum()), stride, pin_memory=True)
    remote[:, :dim] = torch.from_numpy(X)[~is_local]
    cache = B.FeatureCache(n_nodes, 0, stride, DEV)
    cache.loc.copy_(home)
    prep, copy = torch.cuda.Stream(), torch.cuda.Stream()
    sizes = (700, 1, 2500, 0, 64, 4097, 33, 1500)
    batches = [rng.integers(0, n_nodes, size=s).astype(np.int32) for s in sizes]
    nodes_dev = [torch.as_tensor(b, device=DEV) if b.size else torch.empty(1, dtype=torch.int32, device=DEV) for b in batches]
    stats = torch.full((8, 3), -1, dtype=torch.int64, device=DEV)
    outs = [torch.full((max(b.size, 1), stride), float("nan"), device=DEV) for b in batches]
    torch.cuda.synchronize()
    ctx.gather_prepare(0, nodes_dev[:5], sizes[:5], cache, [stats[t] for t in range(5)], stream=prep)
    ctx.gather_prepare(5, nodes_dev[5:], sizes[5:], cache, [stats[t] for t in range(5, 8)], stream=prep,
                       n_dev=[torch.tensor([s], dtype=torch.int32, device=DEV) for s in sizes[5:]])
    done = torch.cuda.Event()
    done.record(prep)
    copy.wait_event(done)
    for t in (2, 7, 0, 3, 6, 1, 5, 4):
        ctx.gather_run(t, sizes[t], cache, local, remote, dim, outs[t], hit_stream=copy)
    torch.cuda.synchronize()
    for t in range(8):
        want, st = oracle.gather_features(X, batches[t], home.numpy())
        assert np.array_equal(outs[t][:sizes[t], :dim].cpu().numpy(), want), t
        assert tuple(stats[t].cpu().tolist()) == st, t
    with pytest.raises(B.RgError) as e:
        ctx.gather_run(1, 5, cache, local, remote, dim, outs[1], hit_stream=copy)      # prepared for 1 row
    assert e.value.status == B.RG_ERR_STATE
    with pytest.raises(B.RgError) as e:
        ctx.gather_prepare(6, nodes_dev[:3], sizes[:3], cache, [stats[t] for t in range(3)])   # tickets 6..8
    assert e.value.status == B.RG_ERR_INVALID_ARG
    # on a fresh context: a batch larger than anything seen so far grows the scratch and drops every earlier preparation
    c2 = B.Context(0)
    c2.gather_prepare(2, [nodes_dev[2]], [sizes[2]], cache, [stats[2]])
    big = rng.integers(0, n_nodes, size=200_000).astype(np.int32)
    c2.gather_prepare(3, [torch.as_tensor(big, device=DEV)], [big.size], cache, [stats[3]])
    with pytest.raises(B.RgError) as e:
        c2.gather_run(2, sizes[2], cache, local, remote, dim, outs[2])
    assert e.value.status == B.RG_ERR_STATE
    out_big = torch.empty(big.size, stride, device=DEV)
    c2.gather_run(3, big.size, cache, local, remote, dim, out_big)
    torch.cuda.synchronize()
    assert np.array_equal(out_big[:, :dim].cpu().numpy(), X[big])
    c2.close()


def test_gather_halves_on_streams_of_their_own(B, ctx):
    """rg_gather_run_part: the HBM-served rows of each batch on one stream, the miss rows on another with the miss halves
    of consecutive batches queued one behind the other (forked once after the lookups, joined per batch), each half
    writing only its own rows; together they give the oracle's rows.  Wrong part values and unprepared tickets are refused."""
    rng = np.random.default_rng(21)
    n_nodes, dim = 5000, 37
    stride = synth.stores.row_stride(dim)
    X = rng.standard_normal((n_nodes, dim)).astype(np.float32)
    is_local = torch.from_numpy(rng.random(n_nodes) < 0.5)
    home = synth.stores.make_home(is_local)
    home_np = home.numpy()
    local = torch.zeros(int(is_local.sum()), stride, device=DEV)
    local[:, :dim] = torch.from_numpy(X)[is_local].to(DEV)
    remote = torch.zeros(int((~is_local).sum()), stride, pin_memory=True)
    remote[:, :dim] = torch.from_numpy(X)[~is_local]
    sizes = (900, 3000, 0, 1, 4097, 64)
    batches = [rng.integers(0, n_nodes, size=k).astype(np.int32) for k in sizes]
    counts_orc = np.zeros(n_nodes, dtype=np.uint32)
    for b in batches:
        oracle.access_histogram(b, counts_orc)
    cap = 400
    ids_orc, loc_orc = oracle.build_cache(counts_orc, home_np, cap)
    counts = torch.as_tensor(counts_orc.view(np.int32), device=DEV)
    cache = B.FeatureCache(n_nodes, cap, stride, DEV)
    ctx.build_cache(counts, home.to(DEV), remote, dim, cache)
    nodes_dev = [torch.as_tensor(b, device=DEV) if b.size else torch.empty(1, dtype=torch.int32, device=DEV) for b in batches]
    stats = torch.full((len(sizes), 3), -1, dtype=torch.int64, device=DEV)
    outs = [torch.full((max(k, 1), stride), float("nan"), device=DEV) for k in sizes]
    rows_s, miss_s = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(rows_s):
        ctx.gather_prepare(0, nodes_dev, sizes, cache, [stats[t] for t in range(len(sizes))])
    ready = torch.cuda.Event()
    ready.record(rows_s)
    miss_s.wait_event(ready)                              # the one fork
    for t, k in enumerate(sizes):                         # every miss half first: they follow each other on their stream
        ctx.gather_run_part(t, B.RG_GATHER_PART_MISS, k, cache, local, remote, dim, outs[t], stream=miss_s)
    miss_s.synchronize()
    want1, st1 = oracle.gather_features(X, batches[1], loc_orc)
    got1 = outs[1][:sizes[1], :dim].cpu().numpy()
    is_miss = ((loc_orc[batches[1]].astype(np.int64) & 0xFFFFFFFF) >> 30) == 2
    assert st1[2] == int(is_miss.sum()) > 0 and np.array_equal(got1[is_miss], want1[is_miss]) and np.isnan(got1[~is_miss]).all()
    for t, k in enumerate(sizes):
        ctx.gather_run_part(t, B.RG_GATHER_PART_HBM, k, cache, local, remote, dim, outs[t], stream=rows_s)
    torch.cuda.synchronize()
    for t, k in enumerate(sizes):
        want, st = oracle.gather_features(X, batches[t], loc_orc)
        assert tuple(stats[t].cpu().tolist()) == st, t
        assert np.array_equal(outs[t][:k, :dim].cpu().numpy(), want), t
    for bad in (0, 3, 4):
        with pytest.raises(B.RgError) as e:
            ctx.gather_run_part(0, bad, sizes[0], cache, local, remote, dim, outs[0])
        assert e.value.status == B.RG_ERR_INVALID_ARG
    with pytest.raises(B.RgError) as e:
        ctx.gather_run_part(0, B.RG_GATHER_PART_MISS, sizes[0] + 1, cache, local, remote, dim, outs[1])
    assert e.value.status == B.RG_ERR_STATE


# ------------------------------------------------------------------------------ histogram
def test_histogram_with_repeats_and_device_count(B, ctx):
    rng = np.random.default_rng(4)
    n_nodes = 1000
    ids = (rng.zipf(1.3, size=200_000) % n_nodes).astype(np.int32)       # heavy repeats
    counts = torch.zeros(n_nodes, dtype=torch.int32, device=DEV)
    ctx.access_histogram(torch.as_tensor(ids, device=DEV), ids.size, counts)
    ctx.access_histogram(torch.as_tensor(ids, device=DEV), ids.size, counts,
                         n_dev=torch.tensor([1234], dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    want = np.zeros(n_nodes, dtype=np.uint32)
    oracle.access_histogram(ids, want)
    oracle.access_histogram(ids[:1234], want)
    assert np.array_equal(counts.cpu().numpy().view(np.uint32), want)


@pytest.mark.parametrize("n_nodes,n_batches", [(100, 0), (100, 1), (8192, 3), (8193, 5), (30_000, 17), (70_000, 40)])
def test_epoch_histogram_matches_per_batch_definition(B, ctx, n_nodes, n_batches):
    """One call over an arena of batches (seed tier unsorted, later tiers ascending, some tiers empty)."""
    log(f"[epoch histogram] N={n_nodes} batches={n_batches}")
    rng = np.random.default_rng(n_nodes + n_batches)
    H, stride, max_seeds = 3, 2048, 16
    arena = np.full((max(n_batches, 1), stride), -1, dtype=np.int32)
    tier_offs = np.zeros((max(n_batches, 1), H + 2), dtype=np.int32)
    want = np.zeros(n_nodes, dtype=np.uint32)
    want[::7] = 3                                            # the call accumulates onto existing counts
    counts = torch.from_numpy(want.view(np.int32).copy()).to(DEV)
    for b in range(n_batches):
        sizes = [int(rng.integers(0, max_seeds + 1))] + [int(rng.integers(0, 600)) if rng.random() < 0.8 else 0 for _ in range(H)]
        sizes = [min(s, n_nodes // 8) for s in sizes]
        ids = rng.permutation(n_nodes)[:sum(sizes)].astype(np.int32)     # unique within a batch
        off = 0
        for t, sz in enumerate(sizes):
            part = ids[off:off + sz]
            arena[b, off:off + sz] = part if t == 0 else np.sort(part)
            off += sz
            tier_offs[b, t + 1] = off
        oracle.access_histogram(arena[b, :off], want)
    ctx.access_histogram_epoch(torch.from_numpy(arena).to(DEV), torch.from_numpy(tier_offs).to(DEV), n_batches, H,
                               max_seeds, counts)
    torch.cuda.synchronize()
    assert np.array_equal(counts.cpu().numpy().view(np.uint32), want)
    # the same call with first-use tracking: counts once more, and the first batch whose list holds each id
    first = torch.full((n_nodes,), -1, dtype=torch.int32, device=DEV)
    first[5] = 0                                             # an earlier period already saw node 5 in batch 0
    ctx.access_histogram_epoch(torch.from_numpy(arena).to(DEV), torch.from_numpy(tier_offs).to(DEV), n_batches, H,
                               max_seeds, counts, first_batch=first)
    torch.cuda.synchronize()
    want2 = want.copy()
    want_first = np.full(n_nodes, 0xFFFFFFFF, dtype=np.uint64)
    want_first[5] = 0
    for b in range(n_batches):
        ids = arena[b, :tier_offs[b, H + 1]]
        oracle.access_histogram(ids, want2)
        want_first[ids] = np.minimum(want_first[ids], b)
    assert np.array_equal(counts.cpu().numpy().view(np.uint32), want2)
    assert np.array_equal(first.cpu().numpy().view(np.uint32).astype(np.uint64), want_first)


# ------------------------------------------------------------------------------ mean aggregation (consumer)
def _agg_tolerance(indptr, nbr, X):
    """fp32 sequential sum of m terms then one division: |error| <= u * (sum|x_e| + |mean|), u = 2^-24
    (standard summation bound (m-1) u sum|x| divided by m, plus the rounding of the division)."""
    m = np.diff(indptr).astype(np.float64)[:, None]
    mean_abs = oracle.mean_aggregate(indptr, nbr, np.abs(X))
    mean = oracle.mean_aggregate(indptr, nbr, X)
    return mean, 1.01 * 2.0 ** -24 * (m * mean_abs + np.abs(mean)) + 1e-37


@pytest.mark.parametrize("dim,pad", [(64, True), (100, True), (256, True), (602, True), (602, False), (7, False), (1, False)])
def test_mean_aggregate_synthetic_segments(B, ctx, dim, pad):
    log(f"[mean aggregate] dim={dim} pad={pad}")
    rng = np.random.default_rng(dim)
    n_dst, n_src = 2500, 6000
    m = rng.integers(0, 12, size=n_dst)
    m[:4] = [0, 1, 100, 33]
    indptr = np.concatenate([[0], np.cumsum(m)]).astype(np.int64)
    nbr = rng.integers(0, n_src, size=int(indptr[-1])).astype(np.int32)
    X = (rng.standard_normal((n_src, dim)) * 10 ** rng.uniform(-3, 3, size=(n_src, 1))).astype(np.float32)
    stride = synth.stores.row_stride(dim) if pad else dim
    feat = torch.zeros(n_src, stride, device=DEV)
    feat[:, :dim] = torch.from_numpy(X).to(DEV)
    agg = torch.full((n_dst, stride), float("nan"), device=DEV)
    ctx.mean_aggregate(torch.as_tensor(indptr.astype(np.int32), device=DEV), torch.as_tensor(nbr, device=DEV), n_dst,
                       feat, dim, agg)
    torch.cuda.synchronize()
    want, tol = _agg_tolerance(indptr, nbr, X)
    got = agg[:, :dim].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - want) <= tol), float(np.max(np.abs(got - want) / tol))
    assert not got[0].any()
    assert np.array_equal(agg[1, :dim].cpu().numpy(), X[nbr[indptr[1]]])      # one neighbour: exact
    # device-side destination count
    agg.fill_(float("nan"))
    ctx.mean_aggregate(torch.as_tensor(indptr.astype(np.int32), device=DEV), torch.as_tensor(nbr, device=DEV), n_dst,
                       feat, dim, agg, n_dst_dev=torch.tensor([1000], dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    got = agg[:, :dim].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got[:1000] - want[:1000]) <= tol[:1000]) and np.isnan(got[1000:]).all()


def test_mean_aggregate_over_sampled_block(B, ctx):
    """Sample a batch, gather its input features, aggregate the outermost hop: the first GraphSAGE layer's AGG."""
    wl = synth.build_workload("small", seed=3, device=DEV)
    cfg = wl.cfg
    H = len(cfg.fanouts)
    rp, ci = host_graph(wl)
    X = wl.features.cpu().numpy()
    csr = B.CsrGraph(wl.row_ptr, wl.col_idx)
    bufs = B.BlockBuffers(cfg.num_nodes, wl.nnz, cfg.batch_size, cfg.fanouts, DEV)
    seeds = wl.train_ids[:cfg.batch_size].contiguous()
    ctx.sample_blocks(csr, seeds, seeds.numel(), cfg.fanouts, wl.seed, 0, bufs)
    torch.cuda.synchronize()
    tier = bufs.tier_off.cpu().tolist()
    n, n_dst = tier[H + 1], tier[H]
    cache = B.FeatureCache(cfg.num_nodes, 0, wl.stride, DEV)
    cache.loc.copy_(wl.home)                                       # no cache: rows come from their home stores
    out = torch.empty(n, wl.stride, device=DEV)
    stats = torch.zeros(3, dtype=torch.int64, device=DEV)
    ctx.gather_features(bufs.nodes, n, cache, wl.local_store, wl.remote_store, cfg.feat_dim, out, stats)
    agg = torch.empty(n_dst, wl.stride, device=DEV)
    ctx.mean_aggregate(bufs.indptr[H - 1], bufs.nbr_local[H - 1], n_dst, out, cfg.feat_dim, agg,
                       n_dst_dev=bufs.tier_off[H:])
    torch.cuda.synchronize()
    blk = oracle.sample_blocks(rp, ci, seeds.cpu().numpy(), cfg.fanouts, wl.seed, 0)
    feats = X[blk.input_nodes]                                     # gathered rows, by the oracle's plain definition
    want, tol = _agg_tolerance(blk.indptr[H - 1], blk.nbr_local[H - 1], feats)
    got = agg[:, :cfg.feat_dim].cpu().numpy().astype(np.float64)
    assert got.shape == want.shape
    assert np.all(np.abs(got - want) <= tol)
    # the same thing written with global ids: mean of X over the sampled neighbours of each frontier node
    i = 17
    nb = blk.nbr[H - 1][blk.indptr[H - 1][i]:blk.indptr[H - 1][i + 1]]
    assert np.allclose(got[i], X[nb].astype(np.float64).mean(0), rtol=1e-5, atol=1e-6)


def test_pipeline_with_mean_consumer_and_output_ring(B):
    """Gathers run up to three batches ahead of the consumer (mean aggregation of the outermost block on its own
    stream) through a ring of output buffers; every batch's aggregate is checked against the oracle."""
    from paper_2505_10806_amd.pipeline import EpochPipeline
    wl = synth.build_workload("tiny", seed=9, device=DEV)
    cfg = wl.cfg
    H = len(cfg.fanouts)
    rp, ci = host_graph(wl)
    X = wl.features.cpu().numpy()
    train_np = wl.train_ids.cpu().numpy()
    pipe = EpochPipeline(wl, device=DEV, consumer="mean", queue_depth=3, double_buffer=True)
    nb = pipe.batches_per_epoch
    blocks = {}

    def epoch_start(p, k):
        p._epoch = k
        for b, seeds in enumerate(oracle.epoch_batches(train_np, cfg.batch_size, wl.seed, k, cfg.max_batches)):
            blocks[(k, b)] = oracle.sample_blocks(rp, ci, seeds, cfg.fanouts, wl.seed, k)

    seen = []

    def batch_done(p, b):
        torch.cuda.synchronize()
        blk = blocks[(p._epoch, b)]
        want, tol = _agg_tolerance(blk.indptr[H - 1], blk.nbr_local[H - 1], X[blk.input_nodes])
        got = p.agg[:want.shape[0], :cfg.feat_dim].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - want) <= tol), f"epoch {p._epoch} batch {b}"
        assert np.array_equal(p.out[:blk.input_nodes.size, :cfg.feat_dim].cpu().numpy(), X[blk.input_nodes])
        seen.append(p.out.data_ptr())

    pipe.run_epochs(0, 2, nb, on_batch=batch_done, on_epoch_start=epoch_start)
    torch.cuda.synchronize()
    assert len(seen) == 2 * nb and len(set(seen)) == 3                      # the ring's three buffers were cycled


def test_kernel_timing_brackets_follow_the_selection(B):
    """rg_profile_*: launches are bracketed only while profiling is on and only for the selected kernel ids; durations
    are positive and the counts are those of the launches made; results are unaffected."""
    wl = synth.build_workload("tiny", seed=6, device=DEV)
    cfg = wl.cfg
    c = B.Context(0)
    X = wl.features.cpu().numpy()
    g = torch.Generator().manual_seed(3)
    nodes = torch.randint(0, cfg.num_nodes, (3000,), generator=g, dtype=torch.int32)
    nodes_dev = nodes.to(DEV)
    counts = torch.zeros(cfg.num_nodes, dtype=torch.int32, device=DEV)
    cache = B.FeatureCache(cfg.num_nodes, wl.capacity_rows, wl.stride, DEV)
    out = torch.zeros(nodes.numel(), wl.stride, device=DEV)
    stats = torch.zeros(3, dtype=torch.int64, device=DEV)

    def work():
        counts.zero_()
        c.access_histogram(nodes_dev, nodes.numel(), counts)
        c.build_cache(counts, wl.home, wl.remote_store, cfg.feat_dim, cache)
        c.gather_features(nodes_dev, nodes.numel(), cache, wl.local_store, wl.remote_store, cfg.feat_dim, out, stats)
        c.gather_features(nodes_dev, nodes.numel(), cache, wl.local_store, wl.remote_store, cfg.feat_dim, out, stats)
        torch.cuda.synchronize()

    def launches():
        return {k: c.profile_read(k) for k in (B.RG_K_GATHER_HBM, B.RG_K_GATHER_MISS, B.RG_K_HISTOGRAM, B.RG_K_CACHE_FILL)}

    work()                                                # profiling off: nothing is recorded
    assert all(n == 0 for _, n in launches().values())
    c.profile_enable(True)
    c.profile_reset()
    work()
    got = launches()
    assert got[B.RG_K_GATHER_HBM][1] == 2 and got[B.RG_K_GATHER_MISS][1] == 2 and got[B.RG_K_HISTOGRAM][1] == 1 and got[B.RG_K_CACHE_FILL][1] == 1
    assert all(ms > 0 for ms, _ in got.values())
    c.profile_select([B.RG_K_GATHER_HBM])                 # this kernel alone
    c.profile_reset()
    work()
    got = launches()
    assert got[B.RG_K_GATHER_HBM][1] == 2 and got[B.RG_K_GATHER_HBM][0] > 0
    assert got[B.RG_K_GATHER_MISS][1] == 0 and got[B.RG_K_HISTOGRAM][1] == 0 and got[B.RG_K_CACHE_FILL][1] == 0
    c.profile_select(None)
    c.profile_enable(False)
    c.profile_reset()
    work()
    assert all(n == 0 for _, n in launches().values())
    counts_orc = np.zeros(cfg.num_nodes, dtype=np.uint32)
    oracle.access_histogram(nodes.numpy(), counts_orc)
    _, loc_orc = oracle.build_cache(counts_orc, wl.home.cpu().numpy(), wl.capacity_rows)
    want, st = oracle.gather_features(X, nodes.numpy(), loc_orc)
    assert tuple(stats.cpu().tolist()) == st and np.array_equal(out[:, :cfg.feat_dim].cpu().numpy(), want)
    c.close()


# ------------------------------------------------------------------------------ argument errors
def test_argument_errors_are_reported_not_launched(B, ctx):
    rp = torch.tensor([0, 1, 2], dtype=torch.int32, device=DEV)
    ci = torch.tensor([1, 0], dtype=torch.int32, device=DEV)
    csr = B.CsrGraph(rp, ci)
    bufs = B.BlockBuffers(2, 2, 2, (2,), DEV)
    seeds = torch.tensor([0, 1], dtype=torch.int32, device=DEV)
    with pytest.raises(B.RgError) as e:
        ctx.sample_blocks(csr, seeds, 2, (B.RG_MAX_FANOUT + 1,), 1, 0, bufs)
    assert e.value.status == B.RG_ERR_INVALID_ARG
    with pytest.raises(B.RgError) as e:
        ctx.sample_blocks(csr, seeds, 2, (-5,), 1, 0, bufs)
    assert e.value.status == B.RG_ERR_INVALID_ARG
    with pytest.raises(B.RgError) as e:
        ctx.sample_blocks(csr, seeds, -1, (2,), 1, 0, bufs)
    assert e.value.status == B.RG_ERR_INVALID_ARG
    small = B.BlockBuffers(2, 2, 1, (2,), DEV)          # sized for one seed, used with two
    assert (small.c_struct.nodes_cap, small._indptr_cap[0], small._nbr_cap[0]) == (2, 2, 2)
    with pytest.raises(B.RgError) as e:
        ctx.sample_blocks(csr, seeds, 2, (2,), 1, 0, small)
    assert e.value.status == B.RG_ERR_CAPACITY
    # the required sizes come back in place of the capacities: frontier bounds [2, 2], edge bound 2
    assert (small.c_struct.nodes_cap, small._indptr_cap[0], small._nbr_cap[0]) == (2, 3, 2)
    assert B.blocks_bounds(2, 2, 2, (2,)) == ([2, 2], [2])
    cache = B.FeatureCache(2, 1, 4, DEV)
    store = torch.zeros(2, 4, device=DEV)
    pinned = torch.zeros(2, 4, pin_memory=True)
    stats = torch.zeros(3, dtype=torch.int64, device=DEV)
    out = torch.zeros(2, 4, device=DEV)
    with pytest.raises(B.RgError) as e:
        ctx.gather_features(seeds, 2, cache, store, pinned, 8, out, stats)      # dim larger than the strides
    assert e.value.status == B.RG_ERR_INVALID_ARG
    with pytest.raises(B.RgError) as e:
        ctx.gather_features(seeds, -3, cache, store, pinned, 4, out, stats)
    assert e.value.status == B.RG_ERR_INVALID_ARG
    with pytest.raises(B.RgError) as e:
        ctx.build_cache(torch.zeros(2, dtype=torch.int32, device=DEV), seeds, pinned, 0, cache)
    assert e.value.status == B.RG_ERR_INVALID_ARG
    # a pageable host pointer as the remote store is refused on the host instead of faulting a kernel
    import ctypes
    pageable = torch.zeros(2, 4)
    st = B._lib.rg_gather_features(ctx._h, seeds.data_ptr(), 2, None, ctypes.byref(cache.c_struct), store.data_ptr(), 4,
                                   pageable.data_ptr(), 4, 4, out.data_ptr(), 4, stats.data_ptr(), None, None)
    assert st == B.RG_ERR_INVALID_ARG and b"not device-accessible" in B._lib.rg_last_error(ctx._h)
    st = B._lib.rg_build_cache(ctx._h, torch.zeros(2, dtype=torch.int32, device=DEV).data_ptr(), seeds.data_ptr(), 2,
                               pageable.data_ptr(), 4, 4, ctypes.byref(cache.c_struct), None)
    assert st == B.RG_ERR_INVALID_ARG
    # the later entry points validate on the host as well
    with pytest.raises(B.RgError) as e:
        ctx.cache_hit_curve(torch.zeros(2, dtype=torch.int32, device=DEV), seeds, [-1])
    assert e.value.status == B.RG_ERR_INVALID_ARG
    plan = B.PrefetchPlan(0, 2, DEV)                       # list too small for the cache's capacity
    with pytest.raises(B.RgError) as e:
        ctx.plan_prefetch(cache, seeds, torch.zeros(2, dtype=torch.int32, device=DEV), plan)
    assert e.value.status == B.RG_ERR_INVALID_ARG
    good_plan = B.PrefetchPlan(1, 2, DEV)
    with pytest.raises(B.RgError) as e:
        ctx.prefetch_planned(good_plan, 4, cache, pinned, 4)   # batch beyond the plan
    assert e.value.status == B.RG_ERR_INVALID_ARG
    with pytest.raises(B.RgError) as e:
        ctx.mean_aggregate(seeds, seeds, 1, store, 8, out)     # dim larger than the strides
    assert e.value.status == B.RG_ERR_INVALID_ARG
    with pytest.raises(B.RgError) as e:
        ctx.access_histogram_epoch(torch.zeros(1, 4, dtype=torch.int32, device=DEV), torch.zeros(1, 11, dtype=torch.int32, device=DEV),
                                   1, 9, 1, torch.zeros(2, dtype=torch.int32, device=DEV))
    assert e.value.status == B.RG_ERR_INVALID_ARG          # more hops than RG_MAX_HOPS
    # the context still works after the rejected calls
    ctx.sample_blocks(csr, seeds, 2, (2,), 1, 0, bufs)
    torch.cuda.synchronize()
    assert bufs.tier_off.cpu().tolist() == [0, 2, 2]
