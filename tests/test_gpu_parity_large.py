"""Parity at the full sizes of the three large workloads, in the launch configuration bench.py times
(EpochPipeline: per-batch arena slots, device-side counts, miss rows on a second stream).

Index outputs are compared bit-exactly with the oracle; gathered rows are compared in full on a subset
of batches (the output is a pure function of the input-node list, which is compared wherever the oracle
is run).  On the stress workload the oracle runs on three batches of the epoch; the whole epoch is then
checked through properties that hold at any size.
"""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_common import HipBatch, assert_batch_equal, host_graph, log

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _tag(words):
    return (np.asarray(words).astype(np.int64) & 0xFFFFFFFF) >> 30


def _compare_block(pipe, B, wl, rp, ci, epoch, slot, seeds_orc, scratch):
    """Oracle block for one batch vs the pipeline's arena slot and a fresh HIP run of the same batch."""
    cfg, H = wl.cfg, len(wl.cfg.fanouts)
    orc = oracle.sample_blocks(rp, ci, seeds_orc, cfg.fanouts, wl.seed, epoch)
    n = int(orc.tier_off[-1])
    assert pipe.tier_offs[slot].cpu().numpy().astype(np.int64).tolist() == orc.tier_off.tolist()
    assert np.array_equal(pipe.arena[slot, :n].cpu().numpy(), orc.nodes)
    pipe.ctx.sample_blocks(pipe.csr, torch.as_tensor(seeds_orc, device=DEV), len(seeds_orc), cfg.fanouts, wl.seed, epoch, scratch)
    assert_batch_equal(HipBatch(scratch, H), orc, H, f"{cfg.name} epoch {epoch} slot {slot}")
    return orc


def _gather_and_compare(pipe, wl, X, X1, slot, nodes_orc, loc_orc, rows, pull=True):
    cfg = wl.cfg
    if not pull:                                        # the cache in use was filled in bulk
        pass
    elif pipe.early_pull:                                 # same order as EpochPipeline.online, synchronous here
        torch.cuda.synchronize()                        # the staging pulls were queued during precompute
        pipe.commit_rows(slot)
    elif pipe.prefetch:
        pipe.prefetch_rows(slot)
    n = pipe.gather(slot)
    torch.cuda.synchronize()
    assert n == nodes_orc.size
    _, st = oracle.gather_features(X1, nodes_orc, loc_orc)            # statistics only (1-column view of X)
    assert tuple(pipe.stats[slot].cpu().tolist()) == st
    if rows:
        want, _ = oracle.gather_features(X, nodes_orc, loc_orc)
        got = pipe.out[:n, :cfg.feat_dim].cpu().numpy()
        assert np.array_equal(got, want), f"gathered rows of slot {slot}"
    return st


def _check_cache_resident(pipe, X, ids_orc, dim):
    """Every selected node was requested by some batch of the period, so after the gathers every slot has
    been pulled exactly once: all resident bits set and every cached row equal to the node's feature row."""
    torch.cuda.synchronize()
    k = ids_orc.size
    bits = pipe.cache.filled.cpu().numpy().view(np.uint32)
    resident = np.unpackbits(bits.view(np.uint8), bitorder="little")[:k]
    assert resident.all(), "a selected slot was never pulled"
    assert not np.unpackbits(bits.view(np.uint8), bitorder="little")[k:].any()
    for lo in range(0, k, 1 << 20):
        hi = min(k, lo + (1 << 20))
        assert np.array_equal(pipe.cache.cache_rows[lo:hi, :dim].cpu().numpy(), X[ids_orc[lo:hi]]), "cached rows"


@pytest.mark.parametrize("name,row_every", [("dense_social", 16), ("sparse_copurchase", 24)])
def test_large_workload_full_epoch(name, row_every):
    from paper_2505_10806_amd import binding as B
    from paper_2505_10806_amd.pipeline import EpochPipeline
    wl = synth.build_workload(name, seed=2025, device=DEV)
    cfg, H = wl.cfg, len(wl.cfg.fanouts)
    log(f"[large] {name}: N={cfg.num_nodes} nnz={wl.nnz} D={cfg.feat_dim} capacity={wl.capacity_rows}")
    rp, ci = host_graph(wl)
    X = wl.features.cpu().numpy()
    X1 = np.ascontiguousarray(X[:, :1])
    home_np, train_np = wl.home.cpu().numpy(), wl.train_ids.cpu().numpy()
    pipe = EpochPipeline(wl, device=DEV)
    scratch = B.BlockBuffers(cfg.num_nodes, wl.nnz, cfg.batch_size, cfg.fanouts, DEV)
    nb = pipe.batches_per_epoch

    # epoch 0: every batch through the oracle; histogram, TopHot, fill and gather statistics in full
    pipe.precompute(0, nb)
    pipe.read_sizes()
    batches = oracle.epoch_batches(train_np, cfg.batch_size, wl.seed, 0)
    assert len(batches) == nb
    counts_orc = np.zeros(cfg.num_nodes, dtype=np.uint32)
    inputs = []
    for b in range(nb):
        orc = _compare_block(pipe, B, wl, rp, ci, 0, b, batches[b], scratch) if b % 8 == 0 or b == nb - 1 else None
        if orc is None:                                   # nodes and tier offsets only (cheaper than a full re-run)
            orc = oracle.sample_blocks(rp, ci, batches[b], cfg.fanouts, wl.seed, 0)
            assert pipe.tier_offs[b].cpu().numpy().astype(np.int64).tolist() == orc.tier_off.tolist()
            assert np.array_equal(pipe.arena[b, :orc.nodes.size].cpu().numpy(), orc.nodes), f"nodes of batch {b}"
        oracle.access_histogram(orc.input_nodes, counts_orc)
        inputs.append(orc.input_nodes)
        if b % 32 == 0:
            log(f"[large] {name} epoch 0 batch {b}/{nb} ok ({orc.nodes.size} input nodes)")
    assert np.array_equal(pipe.counts.cpu().numpy().view(np.uint32), counts_orc), "histogram"
    ids_orc, loc_orc = oracle.build_cache(counts_orc, home_np, wl.capacity_rows)
    k = int(pipe.cache.num_cached.item())
    assert k == ids_orc.size
    assert np.array_equal(pipe.cache.cache_ids[:k].cpu().numpy(), ids_orc)
    assert np.array_equal(pipe.cache.loc.cpu().numpy(), loc_orc)
    tot = np.zeros(3, dtype=np.int64)
    for b in range(nb):
        tot += np.array(_gather_and_compare(pipe, wl, X, X1, b, inputs[b], loc_orc, rows=(b % row_every == 0 or b == nb - 1)))
    _check_cache_resident(pipe, X, ids_orc, cfg.feat_dim)
    remote = _tag(home_np) == 2
    assert tot[1] == int(counts_orc[ids_orc].sum()) and tot[1] + tot[2] == int(counts_orc[remote].sum())
    log(f"[large] {name} epoch 0: cached={k} hit%={100.0 * tot[1] / (tot[1] + tot[2]):.2f} rows={tot.sum()}")

    # epoch 1: a different stream; blocks on a sample of batches
    sample = list(range(0, nb, 37)) + [nb - 1]
    pipe.precompute(1, batch_ids=sample)
    pipe.read_sizes()
    batches1 = oracle.epoch_batches(train_np, cfg.batch_size, wl.seed, 1)
    for slot, b in enumerate(sample):
        orc = _compare_block(pipe, B, wl, rp, ci, 1, slot, batches1[b], scratch)
        assert not np.array_equal(orc.nodes[:cfg.batch_size], inputs[b][:cfg.batch_size])


def test_stress_workload():
    from paper_2505_10806_amd import binding as B
    from paper_2505_10806_amd.pipeline import EpochPipeline
    wl = synth.build_workload("stress", seed=2025, device=DEV)
    cfg, H = wl.cfg, len(wl.cfg.fanouts)
    log(f"[stress] N={cfg.num_nodes} nnz={wl.nnz} D={cfg.feat_dim} capacity={wl.capacity_rows}")
    rp, ci = host_graph(wl)
    X = wl.features.cpu().numpy()
    X1 = np.ascontiguousarray(X[:, :1])
    home_np, train_np = wl.home.cpu().numpy(), wl.train_ids.cpu().numpy()
    pipe = EpochPipeline(wl, device=DEV)
    scratch = B.BlockBuffers(cfg.num_nodes, wl.nnz, cfg.batch_size, cfg.fanouts, DEV)
    nb = pipe.batches_per_epoch
    assert nb == 245
    batches = oracle.epoch_batches(train_np, cfg.batch_size, wl.seed, 0)
    assert len(batches) == nb and len(batches[-1]) == 1_000_000 - 244 * 4096

    # (1) three batches through the oracle: blocks, histogram, TopHot + fill, gather (rows in full)
    sample = [0, 122, nb - 1]
    pipe.precompute(0, batch_ids=sample)
    pipe.read_sizes()
    counts_orc = np.zeros(cfg.num_nodes, dtype=np.uint32)
    inputs = []
    for slot, b in enumerate(sample):
        orc = _compare_block(pipe, B, wl, rp, ci, 0, slot, batches[b], scratch)
        oracle.access_histogram(orc.input_nodes, counts_orc)
        inputs.append(orc.input_nodes)
        log(f"[stress] batch {b}: {orc.nodes.size} input nodes, edges per hop {[int(x.size) for x in orc.nbr]} ok")
    assert np.array_equal(pipe.counts.cpu().numpy().view(np.uint32), counts_orc), "histogram"
    ids_orc, loc_orc = oracle.build_cache(counts_orc, home_np, wl.capacity_rows)
    k = int(pipe.cache.num_cached.item())
    assert k == ids_orc.size == int(((counts_orc > 0) & (_tag(home_np) == 2)).sum())    # capacity exceeds the candidates
    assert np.array_equal(pipe.cache.cache_ids[:k].cpu().numpy(), ids_orc)
    assert np.array_equal(pipe.cache.loc.cpu().numpy(), loc_orc)
    for slot in range(len(sample)):
        st = _gather_and_compare(pipe, wl, X, X1, slot, inputs[slot], loc_orc, rows=True)
        assert st[2] == 0
    _check_cache_resident(pipe, X, ids_orc, cfg.feat_dim)
    log("[stress] three-batch parity ok (all rows served from HBM)")

    # (2) the same three batches with a small cache, so that the miss path runs at full row counts
    small_cap = 100_000
    cache2 = B.FeatureCache(cfg.num_nodes, small_cap, wl.stride, DEV)
    pipe.ctx.build_cache(pipe.counts, wl.home, wl.remote_store, cfg.feat_dim, cache2)
    ids2, loc2 = oracle.build_cache(counts_orc, home_np, small_cap)
    torch.cuda.synchronize()
    assert np.array_equal(cache2.cache_ids[:small_cap].cpu().numpy(), ids2)
    assert np.array_equal(cache2.loc.cpu().numpy(), loc2)
    keep = pipe.cache
    pipe.cache = cache2
    st = _gather_and_compare(pipe, wl, X, X1, 1, inputs[1], loc2, rows=True, pull=False)
    assert st[2] > 100_000
    pipe.cache = keep
    log(f"[stress] small-cache gather ok: local/hit/miss = {st}")

    # (3) the whole epoch as bench.py runs it; properties that hold at any size
    pipe.precompute(0, nb)
    sizes = pipe.read_sizes()
    for slot, b in enumerate(sample):
        assert sizes[b] == inputs[slot].size
        assert np.array_equal(pipe.arena[b, :sizes[b]].cpu().numpy(), inputs[slot])
    counts = pipe.counts.cpu().numpy().view(np.uint32)
    assert int(counts.sum()) == sum(sizes)                                   # histogram total = gathered rows
    assert int(counts.max()) <= nb                                           # ids are unique within a batch
    k = int(pipe.cache.num_cached.item())
    remote = _tag(home_np) == 2
    assert k == int(((counts > 0) & remote).sum())
    cache_ids = pipe.cache.cache_ids[:k].cpu().numpy()
    assert np.all(np.diff(cache_ids) > 0) and np.all(remote[cache_ids]) and np.all(counts[cache_ids] > 0)
    loc = pipe.cache.loc.cpu().numpy()
    assert np.array_equal(loc[cache_ids].astype(np.int64) & 0x3FFFFFFF, np.arange(k))
    pipe.online(nb)                                                          # prefetch stream ahead of the gathers
    torch.cuda.synchronize()
    stats = pipe.stats[:nb].cpu().numpy()
    assert np.array_equal(stats.sum(1), np.array(sizes))
    assert stats[:, 2].sum() == 0 and stats[:, 1].sum() == int(counts[cache_ids].sum())
    assert stats[:, 0].sum() == int(counts[~remote].sum())
    # rows of the last gathered batch against plain indexing of the generated feature matrix
    n_last = sizes[nb - 1]
    got = pipe.out[:n_last, :cfg.feat_dim].cpu().numpy()
    assert np.array_equal(got, X[inputs[2]])
    log(f"[stress] full epoch ok: rows={int(stats.sum())} cached={k}")
