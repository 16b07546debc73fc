"""Parity at the full sizes of the three large workloads, in the launch configuration bench.py times
(EpochPipeline: sampler groups of 8 batches on two lanes writing straight into per-batch buffers, epoch
histogram, TopHot, prefetch plan, classify groups of 8, miss rows on a second stream).

Every batch of every precomputed epoch goes through the oracle, and every index output the grouped sampler
wrote for it is compared bit for bit: nodes, tier offsets, and per hop indptr, nbr, nbr_local and the edge
count; then the epoch's counts, cache ids, location table and each batch's gather statistics.  Gathered rows
are compared in full for every batch of dense_social and sparse_copurchase (both epochs) and, on stress, for
batches {0, every 16th, last} (the rows are a pure function of the input-node list and the location table,
both compared on every batch).  The oracle runs on a few host threads ahead of the comparisons; that only
changes when its results are ready.
"""
import os

import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_common import OracleAhead, host_graph, log

pytestmark = pytest.mark.gpu
PULL_CUS = 16                   # bench.py's default: the launch configuration it times
SEED = int(os.environ.get("RG_TEST_SEED", "2025"))   # master seed of the generated workloads (another graph, split and schedule per value)
DEV = "cuda:0"


def _tag(words):
    return (np.asarray(words).astype(np.int64) & 0xFFFFFFFF) >> 30


def _assert_block_equal(st, b, orc, H, tag):
    """The buffers the grouped sampler wrote for slot b of the epoch state against the oracle's block."""
    tier = st.tier_offs[b].cpu().numpy().astype(np.int64)
    assert tier.tolist() == orc.tier_off.tolist(), f"{tag} tier_off"
    n = int(tier[H + 1])
    assert np.array_equal(st.arena[b, :n].cpu().numpy(), orc.nodes), f"{tag} nodes"
    assert st.edge_counts[b].cpu().tolist() == [int(x.size) for x in orc.nbr], f"{tag} num_edges"
    for h in range(H):
        indptr, nbr, nbr_local = st.blk[h]
        n_h, e = int(tier[h + 1]), int(orc.nbr[h].size)
        assert np.array_equal(indptr[b, :n_h + 1].cpu().numpy().astype(np.int64), orc.indptr[h]), f"{tag} indptr[{h}]"
        assert np.array_equal(nbr[b, :e].cpu().numpy(), orc.nbr[h]), f"{tag} nbr[{h}]"
        assert np.array_equal(nbr_local[b, :e].cpu().numpy(), orc.nbr_local[h]), f"{tag} nbr_local[{h}]"


def _check_cache_resident(pipe, X, ids_orc, dim):
    """Every selected node was requested by some batch of the period, so after the gathers every selected row has
    been pulled exactly once: its resident bit is set, no other is, and the cached row equals the node's feature
    row.  A cached node's row sits at its slot, or at its remote-store row when the cache mirrors the remote store."""
    torch.cuda.synchronize()
    k = ids_orc.size
    bits = pipe.cache.filled.cpu().numpy().view(np.uint32)
    resident = np.unpackbits(bits.view(np.uint8), bitorder="little")
    rows = pipe.cache.rows_of(torch.as_tensor(ids_orc, device=DEV)).cpu().numpy()
    assert pipe.mirror or np.array_equal(rows, np.arange(k))
    assert resident[rows].all(), "a selected row was never pulled"
    assert int(resident.sum()) == k
    for lo in range(0, k, 1 << 20):
        hi = min(k, lo + (1 << 20))
        got = pipe.cache.cache_rows[torch.as_tensor(rows[lo:hi], device=DEV), :dim].cpu().numpy()
        assert np.array_equal(got, X[ids_orc[lo:hi]]), "cached rows"


def _epoch_parity(pipe, wl, host, epoch, row_batches):
    """One whole epoch as bench.py runs it (offline stage, then prefetch stream ahead of the gathers; the pull stream on
    compute units of its own and the caller on the pipeline's work stream), every output against the oracle.
    row_batches: the batches whose gathered rows are compared in full."""
    with torch.cuda.stream(pipe.work_stream):
        return _epoch_parity_on_current_stream(pipe, wl, host, epoch, row_batches)


def _epoch_parity_on_current_stream(pipe, wl, host, epoch, row_batches):
    cfg, H = wl.cfg, len(wl.cfg.fanouts)
    rp, ci, X, X1, home_np, train_np = host
    nb = pipe.batches_per_epoch
    name = cfg.name
    batches = oracle.epoch_batches(train_np, cfg.batch_size, wl.seed, epoch)
    assert len(batches) == nb

    pipe.precompute(epoch, nb)
    sizes = pipe.read_sizes()
    st = pipe.state
    order = oracle.ORDER_FIRST_SEEN if pipe.node_order == 1 else oracle.ORDER_ASCENDING
    ahead = OracleAhead(lambda seeds: oracle.sample_blocks(rp, ci, seeds, cfg.fanouts, wl.seed, epoch, order), batches)
    counts_orc = np.zeros(cfg.num_nodes, dtype=np.uint32)
    inputs = []
    try:
        for b in range(nb):
            orc = ahead.take()
            _assert_block_equal(st, b, orc, H, f"{name} epoch {epoch} batch {b}")
            assert sizes[b] == orc.nodes.size
            oracle.access_histogram(orc.input_nodes, counts_orc)
            inputs.append(orc.input_nodes)
            if b % 32 == 0 or b == nb - 1:
                log(f"[large] {name} epoch {epoch} batch {b}/{nb}: blocks ok ({orc.nodes.size} input nodes, "
                    f"edges per hop {[int(x.size) for x in orc.nbr]})")
    finally:
        ahead.close()
    assert len(batches[-1]) == train_np.size - (nb - 1) * cfg.batch_size          # the partial last batch is a batch

    torch.cuda.synchronize()                    # histogram and TopHot may run on a stream of the pipeline's own
    assert np.array_equal(pipe.counts.cpu().numpy().view(np.uint32), counts_orc), "histogram"
    assert int(counts_orc.sum()) == sum(sizes) and int(counts_orc.max()) <= nb
    ids_orc, loc_orc = oracle.build_cache(counts_orc, home_np, wl.capacity_rows)
    k = int(pipe.cache.num_cached.item())
    assert k == ids_orc.size
    assert np.array_equal(pipe.cache.cache_ids[:k].cpu().numpy(), ids_orc), "cache ids"
    assert np.array_equal(pipe.cache.loc.cpu().numpy(), loc_orc), "location table"
    log(f"[large] {name} epoch {epoch}: histogram and TopHot ok ({k} cached of capacity {wl.capacity_rows})")

    # online stage: pulls ahead on the prefetch stream, one gather per batch; rows and statistics per batch
    row_set = set(row_batches)
    rows_ahead = OracleAhead(lambda b: oracle.gather_features(X, inputs[b], loc_orc)[0], sorted(row_set), workers=4, window=4)
    n_max = max(sizes)
    out_host = torch.empty(n_max, cfg.feat_dim, dtype=torch.float32).pin_memory()
    tot = np.zeros(3, dtype=np.int64)

    def batch_done(p, b):
        torch.cuda.synchronize()
        n = sizes[b]
        _, st_orc = oracle.gather_features(X1, inputs[b], loc_orc)            # statistics only (1-column view of X)
        assert tuple(p.stats[b].cpu().tolist()) == st_orc, f"{name} epoch {epoch} batch {b} statistics"
        tot[:] += np.array(st_orc)
        if b in row_set:
            out_host[:n].copy_(p.out[:n, :cfg.feat_dim])
            want = rows_ahead.take()
            assert np.array_equal(out_host[:n].numpy(), want), f"{name} epoch {epoch} batch {b} gathered rows"
        if b % 32 == 0 or b == nb - 1:
            log(f"[large] {name} epoch {epoch} batch {b}/{nb}: gather ok (local/hit/miss = {st_orc})")

    try:
        pipe.online(nb, on_batch=batch_done)
        torch.cuda.synchronize()
    finally:
        rows_ahead.close()
    _check_cache_resident(pipe, X, ids_orc, cfg.feat_dim)
    remote = _tag(home_np) == 2
    # hits and misses follow exactly from the histogram
    assert tot[1] == int(counts_orc[ids_orc].sum()) and tot[1] + tot[2] == int(counts_orc[remote].sum())
    assert tot[0] == int(counts_orc[~remote].sum()) and int(tot.sum()) == sum(sizes)
    log(f"[large] {name} epoch {epoch}: cached={k} hit%={100.0 * tot[1] / max(1, tot[1] + tot[2]):.2f} rows={int(tot.sum())} "
        f"(rows compared in full on {len(row_set)} of {nb} batches)")
    return inputs, tot


def _host_inputs(wl):
    rp, ci = host_graph(wl)
    X = wl.features.cpu().numpy()
    X1 = np.ascontiguousarray(X[:, :1])
    return rp, ci, X, X1, wl.home.cpu().numpy(), wl.train_ids.cpu().numpy()


@pytest.mark.parametrize("name", ["dense_social", "sparse_copurchase"])
def test_large_workload_both_epochs(name):
    from paper_2505_10806_amd.pipeline import EpochPipeline
    wl = synth.build_workload(name, seed=SEED, device=DEV)
    cfg = wl.cfg
    log(f"[large] {name}: N={cfg.num_nodes} nnz={wl.nnz} D={cfg.feat_dim} capacity={wl.capacity_rows}")
    host = _host_inputs(wl)
    pipe = EpochPipeline(wl, device=DEV, keep_blocks=True, pull_cus=PULL_CUS)
    nb = pipe.batches_per_epoch
    assert cfg.epochs == 2
    first = None
    for epoch in range(cfg.epochs):
        inputs, tot = _epoch_parity(pipe, wl, host, epoch, range(nb))
        assert tot[2] > 0                                                    # the miss path ran at full size
        if first is None:
            first = inputs[0][:cfg.batch_size].copy()
        else:
            assert not np.array_equal(first, inputs[0][:cfg.batch_size])    # the second epoch has its own schedule


def test_large_workload_first_seen_order_and_bitmap_counts():
    """The second canonical node order at full size, with the access counts (and the first batch of every node, which
    drives the prefetch plan) taken straight from the sampler's membership bitmaps: one epoch of sparse_copurchase."""
    from paper_2505_10806_amd.pipeline import EpochPipeline
    wl = synth.build_workload("sparse_copurchase", seed=SEED, device=DEV)
    host = _host_inputs(wl)
    pipe = EpochPipeline(wl, device=DEV, keep_blocks=True, node_order="first_seen", histogram="sampled", pull_cus=PULL_CUS)
    assert pipe.planned
    nb = pipe.batches_per_epoch
    inputs, tot = _epoch_parity(pipe, wl, host, 0, range(0, nb, 4))
    assert tot[2] > 0
    # the tiers really are in another order than ascending somewhere
    H = len(wl.cfg.fanouts)
    tier = pipe.tier_offs[0].cpu().numpy()
    last = pipe.arena[0, tier[H]:tier[H + 1]].cpu().numpy()
    assert np.any(np.diff(last) < 0)


def test_stress_workload():
    from paper_2505_10806_amd import binding as B
    from paper_2505_10806_amd.pipeline import EpochPipeline
    wl = synth.build_workload("stress", seed=SEED, device=DEV)
    cfg = wl.cfg
    log(f"[stress] N={cfg.num_nodes} nnz={wl.nnz} D={cfg.feat_dim} capacity={wl.capacity_rows}")
    host = _host_inputs(wl)
    rp, ci, X, X1, home_np, train_np = host
    pipe = EpochPipeline(wl, device=DEV, keep_blocks=True, pull_cus=PULL_CUS)
    nb = pipe.batches_per_epoch
    assert nb == 245 and train_np.size == 1_000_000

    # (1) the whole epoch; gathered rows on batches {0, every 16th, last}
    row_batches = sorted(set(range(0, nb, 16)) | {nb - 1})
    inputs, tot = _epoch_parity(pipe, wl, host, 0, row_batches)
    assert tot[2] == 0                                # the cache holds every accessed remote row: all rows come from HBM
    counts = pipe.counts.cpu().numpy().view(np.uint32)
    assert int(pipe.cache.num_cached.item()) == int(((counts > 0) & (_tag(home_np) == 2)).sum())

    # (2) one batch with a small cache, so that the miss path runs at this row count and row length as well
    small_cap = 100_000
    cache2 = B.FeatureCache(cfg.num_nodes, small_cap, wl.stride, DEV)
    pipe.ctx.build_cache(pipe.counts, wl.home, wl.remote_store, cfg.feat_dim, cache2)
    ids2, loc2 = oracle.build_cache(counts, home_np, small_cap)
    torch.cuda.synchronize()
    assert np.array_equal(cache2.cache_ids[:small_cap].cpu().numpy(), ids2)
    assert np.array_equal(cache2.loc.cpu().numpy(), loc2)
    b = 122
    n = inputs[b].size
    stats = torch.zeros(3, dtype=torch.int64, device=DEV)
    pipe.ctx.gather_features(pipe.arena[b], n, cache2, wl.local_store, wl.remote_store, cfg.feat_dim, pipe.out, stats,
                             miss_stream=pipe.side)
    torch.cuda.synchronize()
    want, st_orc = oracle.gather_features(X, inputs[b], loc2)
    assert tuple(stats.cpu().tolist()) == st_orc and st_orc[2] > 100_000
    assert np.array_equal(pipe.out[:n, :cfg.feat_dim].cpu().numpy(), want)
    log(f"[stress] small-cache gather ok: local/hit/miss = {st_orc}")

    # (3) the same epoch once more, the way bench.py runs it: run_epoch from a cold cache with no host synchronisation
    # between the batches (one pull per sampler call, its rows listed from the sampler's bitmaps).  Statistics of every
    # batch against those verified in (1), rows of a few batches against the features of the oracle's input nodes.
    assert pipe.mirror and pipe.group_pulls
    stats1 = pipe.stats[:nb].clone()
    ids1 = pipe.cache.cache_ids.clone()
    loc1 = pipe.cache.loc.clone()
    pipe.stats.zero_()
    pipe.cache.cache_rows.fill_(float("nan"))
    keep = {0: None, 1: None, 9: None, 130: None, nb - 1: None}
    sizes_seen = []

    def capture(p, b):
        sizes_seen.append(p.sizes[b])
        if b in keep:
            keep[b] = p.out[:p.sizes[b], :cfg.feat_dim].clone()

    log("[stress] second pass: start")
    with torch.cuda.stream(pipe.work_stream):
        pipe.run_epoch(0, nb, on_batch=capture)
    torch.cuda.synchronize()
    assert sizes_seen == [x.size for x in inputs]
    assert torch.equal(pipe.stats[:nb], stats1), "statistics of the second pass"
    assert torch.equal(pipe.cache.cache_ids, ids1) and torch.equal(pipe.cache.loc, loc1)
    for b, rows in keep.items():
        assert np.array_equal(rows.cpu().numpy(), X[inputs[b]]), f"second pass batch {b} gathered rows"
    ids_orc = ids1[:int(pipe.cache.num_cached.item())].cpu().numpy()
    _check_cache_resident(pipe, X, ids_orc, cfg.feat_dim)
    log("[stress] second pass ok")
