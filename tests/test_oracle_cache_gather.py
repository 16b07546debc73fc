"""Pins for the oracle's histogram, TopHot cache selection, cache fill and gather (CPU only)."""
import os

import numpy as np
import pytest

import oracle
import synth
from synth import TAG_CACHE, TAG_LOCAL, TAG_REMOTE, TAG_SHIFT, ROW_MASK


def _tag(words):
    return (np.asarray(words).astype(np.int64) & 0xFFFFFFFF) >> TAG_SHIFT


def _row(words):
    return (np.asarray(words).astype(np.int64) & 0xFFFFFFFF) & ROW_MASK


def test_histogram_is_bincount_and_accumulates():
    rng = np.random.default_rng(0)
    n = 5000
    a = rng.integers(0, n, size=40_000).astype(np.int32)
    b = rng.integers(0, 50, size=10_000).astype(np.int32)
    counts = np.zeros(n, dtype=np.uint32)
    oracle.access_histogram(a, counts)
    assert np.array_equal(counts, np.bincount(a, minlength=n).astype(np.uint32))
    oracle.access_histogram(b, counts)
    assert np.array_equal(counts, (np.bincount(a, minlength=n) + np.bincount(b, minlength=n)).astype(np.uint32))
    assert counts.sum() == a.size + b.size
    oracle.access_histogram(np.empty(0, dtype=np.int32), counts)
    assert counts.sum() == a.size + b.size


def _topk_bruteforce(counts, home, capacity):
    ids = np.flatnonzero((_tag(home) == TAG_REMOTE) & (counts >= 1))
    order = ids[np.lexsort((ids, -counts[ids].astype(np.int64)))]      # count desc, then id asc
    chosen = np.sort(order[:max(0, min(capacity, order.size))])
    loc = home.copy().astype(np.int64) & 0xFFFFFFFF
    loc[chosen] = (TAG_CACHE << TAG_SHIFT) | np.arange(chosen.size)
    return chosen, loc


@pytest.mark.parametrize("capacity", [0, 1, 7, 100, 399, 400, 401, 10_000])
def test_topk_matches_full_sort(capacity):
    rng = np.random.default_rng(capacity)
    n = 3000
    is_local = torch_mask(n, rng)
    home = synth.stores.make_home(is_local).numpy()
    counts = rng.integers(0, 6, size=n).astype(np.uint32)           # many ties, many zeros
    counts[rng.integers(0, n, 5)] = 2 ** 31 + 5                     # counts above 2^31 order correctly
    ids, loc = oracle.build_cache(counts, home, capacity)
    want_ids, want_loc = _topk_bruteforce(counts, home, capacity)
    assert ids.tolist() == want_ids.tolist()
    assert np.array_equal(loc.astype(np.int64) & 0xFFFFFFFF, want_loc)
    # invariants
    cand = np.flatnonzero((_tag(home) == TAG_REMOTE) & (counts >= 1))
    assert ids.size == min(capacity, cand.size)
    assert np.all(np.diff(ids) > 0)
    assert np.all(_tag(home[ids]) == TAG_REMOTE) and np.all(counts[ids] >= 1)
    outside = np.setdiff1d(cand, ids)
    if ids.size and outside.size:
        worst_in = min((int(counts[v]), -int(v)) for v in ids)
        best_out = max((int(counts[v]), -int(v)) for v in outside)
        assert worst_in > best_out
    assert np.array_equal(_row(loc[ids]), np.arange(ids.size))
    rest = np.setdiff1d(np.arange(n), ids)
    assert np.array_equal(loc[rest], home[rest])


def torch_mask(n, rng):
    import torch
    return torch.from_numpy(rng.random(n) < 0.3)


def test_topk_ties_break_to_lower_id():
    import torch
    home = synth.stores.make_home(torch.zeros(10, dtype=torch.bool)).numpy()    # all remote
    counts = np.array([2, 5, 2, 2, 0, 5, 2, 1, 2, 2], dtype=np.uint32)
    ids, _ = oracle.build_cache(counts, home, 4)
    assert ids.tolist() == [0, 1, 2, 5]                   # both 5s, then the two lowest ids with count 2
    ids, _ = oracle.build_cache(counts, home, 100)
    assert ids.tolist() == [0, 1, 2, 3, 5, 6, 7, 8, 9]     # never caches the zero-count node


def test_gather_is_plain_indexing_and_hit_rate_closed_form():
    wl = synth.build_workload("tiny", seed=7)
    cfg = wl.cfg
    X = wl.features.numpy()
    rp = wl.row_ptr.numpy().astype(np.int64)
    ci = wl.col_idx.numpy()
    home = wl.home.numpy()
    counts = np.zeros(cfg.num_nodes, dtype=np.uint32)
    batches = oracle.epoch_batches(wl.train_ids.numpy(), cfg.batch_size, wl.seed, 0, cfg.max_batches)
    assert len(batches) == 4
    inputs = []
    for seeds in batches:
        blk = oracle.sample_blocks(rp, ci, seeds, cfg.fanouts, wl.seed, 0)
        inputs.append(blk.input_nodes)
        oracle.access_histogram(blk.input_nodes, counts)
    assert counts.sum() == sum(x.size for x in inputs)                       # (d) totals
    assert counts.max() <= len(batches)                                      # ids unique per batch
    ids, loc = oracle.build_cache(counts, home, wl.capacity_rows)
    assert wl.capacity_rows == 500 and ids.size == 500
    rows = oracle.fill_cache(X, ids, wl.stride)
    assert np.array_equal(rows[:, :cfg.feat_dim], X[ids])
    # the packed stores hold the same rows the location words point at
    loc_u = loc.astype(np.int64) & 0xFFFFFFFF
    local_rows = wl.local_store.numpy()
    remote_rows = wl.remote_store.numpy()
    for v in (0, 1, 2, 3, 4999, 9998, 9999):
        store = local_rows if _tag(home[v]) == TAG_LOCAL else remote_rows
        assert np.array_equal(store[_row(home[v]), :cfg.feat_dim], X[v])
    tot_hit = tot_miss = tot_local = 0
    for nodes in inputs:
        out, (n_local, n_hit, n_miss) = oracle.gather_features(X, nodes, loc, wl.stride)
        assert np.array_equal(out[:, :cfg.feat_dim], X[nodes])
        assert n_local + n_hit + n_miss == nodes.size
        tags = loc_u[nodes] >> TAG_SHIFT
        assert (n_local, n_hit, n_miss) == tuple(int((tags == t).sum()) for t in (TAG_LOCAL, TAG_CACHE, TAG_REMOTE))
        tot_local += n_local
        tot_hit += n_hit
        tot_miss += n_miss
    remote = _tag(home) == TAG_REMOTE
    assert tot_hit == int(counts[ids].sum())                                 # hits predicted by the histogram
    assert tot_hit + tot_miss == int(counts[remote].sum())
    assert tot_local == int(counts[~remote].sum())
    assert 0 < tot_hit < tot_hit + tot_miss


def test_miss_bytes_follow_paper_accounting(golden_dir):
    """Remote rows fetched * 4*D bytes reproduces the figures the paper prints."""
    kv = {}
    with open(os.path.join(golden_dir, "paper_byte_accounting.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                kv[k] = float(v)

    def miss_bytes(n_miss, dim):
        return n_miss * 4 * dim
    assert miss_bytes(kv["remote_rows_per_batch"], kv["feature_tensor_dim"]) == kv["per_batch_bytes"]
    assert round(kv["per_batch_bytes"] / 2 ** 20, 2) == kv["per_batch_mib"]
    assert round(kv["batches_per_epoch"] * kv["per_batch_bytes"] / 1e9, 1) == kv["epoch_gb"]
    assert round(miss_bytes(kv["table4_rows_rapidgnn"], kv["table4_dim"]) / 2 ** 20) == kv["table4_mb_rapidgnn"]
    assert round(miss_bytes(kv["table4_rows_baseline"], kv["table4_dim"]) / 2 ** 20) == kv["table4_mb_baseline"]


def test_mean_aggregate_is_normalised_sparse_product():
    """Mean aggregation = (D^-1 A) X for the block's 0/1 incidence matrix A: checked against scipy's float64
    sparse product, plus the closed forms for one neighbour, no neighbour and identical sources."""
    import scipy.sparse as sp
    rng = np.random.default_rng(2)
    n_dst, n_src, dim = 300, 900, 37
    m = rng.integers(0, 8, size=n_dst)
    m[:5] = [0, 1, 1, 0, 7]
    indptr = np.concatenate([[0], np.cumsum(m)]).astype(np.int64)
    nbr = rng.integers(0, n_src, size=int(indptr[-1])).astype(np.int32)      # repeats allowed
    X = rng.standard_normal((n_src, dim)).astype(np.float32)
    got = oracle.mean_aggregate(indptr, nbr, X)
    A = sp.csr_matrix((np.ones(nbr.size), nbr, indptr), shape=(n_dst, n_src))
    inv = np.divide(1.0, m, out=np.zeros(n_dst), where=m > 0)
    want = sp.diags(inv) @ (A @ X.astype(np.float64))
    assert np.allclose(got, want, rtol=1e-13, atol=1e-13)
    assert not got[0].any() and not got[3].any()                             # no sampled neighbour -> zero row
    assert np.array_equal(got[1], X[nbr[indptr[1]]].astype(np.float64))      # one neighbour -> that row
    same = oracle.mean_aggregate(np.array([0, 4]), np.array([9, 9, 9, 9], dtype=np.int32), X)
    assert np.array_equal(same[0], X[9].astype(np.float64))
    # transposed operand / wrong normaliser would fail this: two destinations sharing sources in different order
    two = oracle.mean_aggregate(np.array([0, 2, 5]), np.array([1, 2, 2, 1, 3], dtype=np.int32), X)
    assert np.allclose(two[0], (X[1].astype(np.float64) + X[2]) / 2) and np.allclose(two[1], (X[2].astype(np.float64) + X[1] + X[3]) / 3)


def test_hit_curve_equals_hits_of_built_caches():
    """hits(K) must equal the cache hits actually counted when a cache of capacity K is built and every batch of
    the period is gathered; it is non-decreasing, concave, and saturates at the total of remote requests."""
    wl = synth.build_workload("tiny", seed=13)
    cfg = wl.cfg
    X = wl.features.numpy()
    rp, ci = wl.row_ptr.numpy().astype(np.int64), wl.col_idx.numpy()
    home = wl.home.numpy()
    counts = np.zeros(cfg.num_nodes, dtype=np.uint32)
    inputs = []
    for seeds in oracle.epoch_batches(wl.train_ids.numpy(), cfg.batch_size, wl.seed, 0, 4):
        blk = oracle.sample_blocks(rp, ci, seeds, cfg.fanouts, wl.seed, 0)
        oracle.access_histogram(blk.input_nodes, counts)
        inputs.append(blk.input_nodes)
    caps = [0, 1, 10, 100, 500, 1000, 2500, 5000, 10 ** 6]
    hits, total = oracle.cache_hit_curve(counts, home, caps)
    remote = _tag(home) == TAG_REMOTE
    assert total == int(counts[remote].sum())
    for k, h in zip(caps, hits):
        _, loc = oracle.build_cache(counts, home, k)
        served = sum(oracle.gather_features(X[:, :1].copy(), nodes, loc)[1][1] for nodes in inputs)
        assert int(h) == served, k
    assert hits[0] == 0 and int(hits[-1]) == total
    dense_caps = np.arange(0, 3000)
    h = oracle.cache_hit_curve(counts, home, dense_caps)[0].astype(np.int64)
    assert np.all(np.diff(h) >= 0) and np.all(np.diff(h, 2) <= 0)            # sorted counts: concave prefix sums
