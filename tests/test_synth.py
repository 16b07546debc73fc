"""The seeded input generators: shapes, encodings and determinism (CPU only)."""
import numpy as np
import pytest
import torch

import synth
from synth import TAG_LOCAL, TAG_REMOTE, TAG_SHIFT, ROW_MASK


def test_configs_match_the_five_workloads():
    assert sorted(synth.CONFIGS) == ["dense_social", "small", "sparse_copurchase", "stress", "tiny"]
    c = synth.get_config("stress")
    assert (c.num_nodes, c.feat_dim, c.fanouts, c.batch_size, c.offsets64) == (10_000_000, 256, (15, 10, 5), 4096, True)
    assert c.cache_capacity_rows(7_500_000) == 48_000_000_000 // 1024
    assert synth.get_config("dense_social").cache_capacity_rows(174_723) == 34_944       # floor(0.20 * remote)
    assert synth.get_config("tiny").tier_upper_bounds() == [256, 2816, 10_000]
    assert c.tier_upper_bounds() == [4096, 65_536, 720_896, 4_325_376]
    with pytest.raises(KeyError):
        synth.get_config("nope")


def test_static_bounds_agree_with_the_library():
    from paper_2505_10806_amd import binding
    for name, cfg in synth.CONFIGS.items():
        nnz = int(cfg.mean_degree * cfg.num_nodes)
        fub, _ = binding.blocks_bounds(cfg.num_nodes, nnz, cfg.batch_size, cfg.fanouts)
        assert all(a <= b for a, b in zip(fub, cfg.tier_upper_bounds())), name
        assert fub[0] == cfg.batch_size


def test_workload_is_reproducible_and_consistent():
    a = synth.build_workload("tiny", seed=77)
    b = synth.build_workload("tiny", seed=77)
    c = synth.build_workload("tiny", seed=78)
    for x, y in [(a.row_ptr, b.row_ptr), (a.col_idx, b.col_idx), (a.features, b.features), (a.train_ids, b.train_ids),
                 (a.home, b.home), (a.local_store, b.local_store), (a.remote_store, b.remote_store)]:
        assert torch.equal(x, y)
    assert not torch.equal(a.col_idx, c.col_idx) and not torch.equal(a.features, c.features)
    cfg = a.cfg
    n = cfg.num_nodes
    assert a.row_ptr.numel() == n + 1 and int(a.row_ptr[-1]) == a.col_idx.numel()
    assert 0.9 * cfg.mean_degree * n <= a.nnz <= cfg.mean_degree * n          # a few % lost to duplicates
    assert a.train_ids.numel() == int(cfg.train_frac * n) and a.train_ids.unique().numel() == a.train_ids.numel()
    assert a.batches_per_epoch() == cfg.max_batches == 4
    assert a.n_local + a.n_remote == n and a.capacity_rows == int(cfg.cache_frac * a.n_remote)
    # location words: tag and packed row, ascending by id inside each store
    w = a.home.numpy().astype(np.int64) & 0xFFFFFFFF
    tag, row = w >> TAG_SHIFT, w & ROW_MASK
    is_local = a.is_local.numpy()
    assert np.array_equal(tag == TAG_LOCAL, is_local) and np.array_equal(tag == TAG_REMOTE, ~is_local)
    assert np.array_equal(row[is_local], np.arange(a.n_local)) and np.array_equal(row[~is_local], np.arange(a.n_remote))
    X = a.features.numpy()
    assert np.array_equal(a.local_store.numpy()[:, :cfg.feat_dim], X[is_local])
    assert np.array_equal(a.remote_store.numpy()[:, :cfg.feat_dim], X[~is_local])
    assert a.stride == synth.stores.row_stride(cfg.feat_dim) == 64


def test_row_stride_pads_to_sixteen_bytes():
    assert [synth.stores.row_stride(d) for d in (1, 4, 100, 602, 603, 604)] == [4, 4, 100, 604, 604, 604]


def test_partitions():
    assert synth.make_partition(8, "mod2", 0).tolist() == [True, False] * 4
    assert synth.make_partition(8, "mod4", 0).tolist() == [True, False, False, False] * 2
    r = synth.make_partition(100_000, "random4", 5)
    assert abs(float(r.float().mean()) - 0.25) < 0.01
    assert torch.equal(r, synth.make_partition(100_000, "random4", 5))
    with pytest.raises(ValueError):
        synth.make_partition(8, "metis", 0)


def test_planted_groups_and_group_partition():
    """The two extra presets share one graph; along the planted groups far fewer edges of local nodes leave the
    partition than under a random partition, and the seeds come from the local partition."""
    assert sorted(synth.EXTRA_CONFIGS) == ["small_groups_local", "small_groups_random"]
    import dataclasses
    small = {k: dataclasses.replace(synth.get_config(k), num_nodes=20_000) for k in synth.EXTRA_CONFIGS}
    r = synth.build_workload(small["small_groups_random"], seed=9)
    g = synth.build_workload(small["small_groups_local"], seed=9)
    assert torch.equal(r.row_ptr, g.row_ptr) and torch.equal(r.col_idx, g.col_idx)
    assert g.n_local == 5_000 and abs(r.n_local - 5_000) < 300

    def leaving(wl):
        rp, ci, loc = wl.row_ptr.numpy(), wl.col_idx.numpy(), wl.is_local.numpy()
        src = np.repeat(np.arange(rp.size - 1), np.diff(rp))
        return (loc[src] & ~loc[ci]).sum() / loc[src].sum()
    assert leaving(r) > 0.7 and leaving(g) < 0.2
    for wl in (r, g):
        assert bool(wl.is_local[wl.train_ids.long()].all()) and wl.train_ids.numel() > 2_000
    # graphs without planted groups are what they were before the option existed
    rp, ci = synth.chung_lu_csr(3000, 10, 2.1, seed=4)
    rp2, ci2, labels = synth.chung_lu_csr(3000, 10, 2.1, seed=4, communities=0, return_communities=True)
    assert labels is None and torch.equal(rp, rp2) and torch.equal(ci, ci2)
