"""The oracle's pins must notice plausible mistakes: each mutant below is the oracle source with one
small error planted (a wrong constant, sign, index, comparison or operand), compiled on the CPU into a
throw-away library and run against a compact version of the pins.  Every mutant has to fail at least
one of them; the unmodified source has to pass them all.  Nothing here touches the GPU.
"""
import itertools
import os
import subprocess
from collections import Counter

import numpy as np
import pytest

import synth

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "rg_oracle.c")
HDR_DIR = os.path.join(os.path.dirname(HERE), "oracle")

# (name, text in rg_oracle.c, replacement)
MUTANTS = [
    ("philox_multiplier", "0xD2511F53u * (uint64_t)c0", "0xD2511F55u * (uint64_t)c0"),
    ("philox_swapped_products", "uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;", "uint32_t n0 = (uint32_t)(p0 >> 32) ^ c1 ^ k0;"),
    ("philox_nine_rounds", "round < 10", "round < 9"),
    ("philox_key_not_bumped", "k1 += 0xBB67AE85u;", ""),
    ("draw_block_index", "(uint32_t)(i >> 2), epoch", "(uint32_t)(i >> 1), epoch"),
    ("draw_word_index", "return out[i & 3];", "return out[(i + 1) & 3];"),
    ("draw_ignores_epoch", "(uint32_t)(i >> 2), epoch }", "(uint32_t)(i >> 2), 0u }"),
    ("draw_ignores_seed_high", "(uint32_t)(seed >> 32) };\n    uint32_t out[4];", "0u };\n    uint32_t out[4];"),
    ("floyd_swapped_branches", "pos[i] = present ? j : t;", "pos[i] = present ? t : j;"),
    ("floyd_range_off_by_one", "(r * (uint64_t)(j + 1)) >> 32", "(r * (uint64_t)(j)) >> 32"),
    ("floyd_wrong_j", "int64_t j = d - k + i;", "int64_t j = d - k + i - 1;"),
    ("floyd_no_membership_test", "if (pos[l] == t) present = 1;", "if (pos[l] == t) present = 0;"),
    # (d < k instead of d <= k is an equivalent program: at d == k Floyd's step i can only produce position i,
    # so the whole row comes out in row order either way; it is therefore not listed)
    ("schedule_key_words_swapped", "((uint64_t)w[0] << 32) | (uint64_t)w[1]", "((uint64_t)w[1] << 32) | (uint64_t)w[0]"),
    ("schedule_hop_marker", "0xFFFFFFFFu, 0u, epoch };\n        uint32_t w[4];", "0u, 0u, epoch };\n        uint32_t w[4];"),
    ("blocks_hop_stream", "(uint32_t)v, (uint32_t)h, d, k, pos)", "(uint32_t)v, 0u, d, k, pos)"),
    ("blocks_tier_not_deduplicated", "if (e == 0 || fresh[e] != fresh[e - 1]) fresh[n_unique++] = fresh[e];", "fresh[n_unique++] = fresh[e];"),
    ("blocks_tier_includes_members", "if (where[nbr[e]] < 0) fresh[n_fresh++] = nbr[e];", "fresh[n_fresh++] = nbr[e];"),
    ("blocks_first_seen_keeps_repeats", "if (where[u] < 0) {\n                    nodes[n] = u;\n                    where[u] = n;", "if (where[u] < 0 || where[u] >= n_h) {\n                    nodes[n] = u;\n                    where[u] = n;"),
    ("blocks_first_seen_walks_backwards", "for (int64_t e = 0; e < E; ++e) {\n                int32_t u = nbr[e];", "for (int64_t e = E - 1; e >= 0; --e) {\n                int32_t u = nbr[e];"),
    ("blocks_row_offset", "col_idx[row_ptr[v] + pos[t]]", "col_idx[row_ptr[v + 1] - 1 - pos[t]]"),
    ("histogram_skips_repeats", "counts[nodes[i]] += 1u;", "counts[nodes[i]] = 1u;"),
    ("tophot_ascending_counts", "return x->count > y->count ? -1 : 1;   /* larger count first */", "return x->count < y->count ? -1 : 1;"),
    ("tophot_ties_to_higher_id", "return x->id < y->id ? -1 : 1;               /* then lower id */", "return x->id > y->id ? -1 : 1;"),
    ("tophot_caches_local", "if (tag == ORC_TAG_REMOTE && counts[v] >= 1u) {\n            cand[n_cand].count = counts[v];\n            cand[n_cand].id = (int32_t)v;\n            ++n_cand;\n        }\n    }\n    qsort(cand, (size_t)n_cand, sizeof(orc_cand), orc_cand_cmp);\n    int64_t k_eff",
     "if (counts[v] >= 1u) {\n            cand[n_cand].count = counts[v];\n            cand[n_cand].id = (int32_t)v;\n            ++n_cand;\n        }\n    }\n    qsort(cand, (size_t)n_cand, sizeof(orc_cand), orc_cand_cmp);\n    int64_t k_eff"),
    ("tophot_caches_untouched", "tag == ORC_TAG_REMOTE && counts[v] >= 1u) {\n            cand[n_cand].count = counts[v];\n            cand[n_cand].id = (int32_t)v;\n            ++n_cand;\n        }\n    }\n    qsort(cand, (size_t)n_cand, sizeof(orc_cand), orc_cand_cmp);\n    int64_t k_eff",
     "tag == ORC_TAG_REMOTE) {\n            cand[n_cand].count = counts[v];\n            cand[n_cand].id = (int32_t)v;\n            ++n_cand;\n        }\n    }\n    qsort(cand, (size_t)n_cand, sizeof(orc_cand), orc_cand_cmp);\n    int64_t k_eff"),
    ("gather_wrong_row", "out[i * out_stride + c] = X[v * dim + c];", "out[i * out_stride + c] = X[(int64_t)i * dim + c];"),
    ("gather_stats_swapped", "if (tag == ORC_TAG_LOCAL) stats[0] += 1;\n        else if (tag == ORC_TAG_CACHE) stats[1] += 1;", "if (tag == ORC_TAG_LOCAL) stats[1] += 1;\n        else if (tag == ORC_TAG_CACHE) stats[0] += 1;"),
    ("fill_wrong_source", "X[(int64_t)cache_ids[s] * dim + c]", "X[(int64_t)s * dim + c]"),
    ("mean_divides_by_dim", "m > 0 ? sum / (double)m : 0.0", "m > 0 ? sum / (double)dim : 0.0"),
    ("hit_curve_counts_rows", "sum += cand[s].count;\n        hits[j] = sum;", "sum += 1;\n        hits[j] = sum;"),
]


def _build(tmp_path, name, old=None, new=None):
    text = open(SRC).read()
    if old is not None:
        assert text.count(old) == 1, f"mutant {name}: pattern occurs {text.count(old)} times"
        text = text.replace(old, new)
    c_path = os.path.join(tmp_path, f"{name}.c")
    so_path = os.path.join(tmp_path, f"{name}.so")
    open(c_path, "w").write(text)
    subprocess.run(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-w", "-I", HDR_DIR, "-o", so_path, c_path], check=True)
    return so_path


class _Lib:
    """The oracle's Python front end bound to another shared library."""

    def __init__(self, so_path):
        import oracle
        self.mod = oracle
        self.saved = (oracle._lib, oracle._LIB_PATH)
        oracle._lib, oracle._LIB_PATH = None, so_path
        real_build = oracle.build
        oracle.build = lambda force=False: so_path
        try:
            oracle.lib()
        finally:
            oracle.build = real_build

    def close(self):
        self.mod._lib, self.mod._LIB_PATH = self.saved


@pytest.fixture(scope="module")
def workload():
    wl = synth.build_workload("tiny", seed=31)
    return wl, wl.row_ptr.numpy().astype(np.int64), wl.col_idx.numpy(), wl.features.numpy(), wl.home.numpy()


def _compact_pins(orc, workload):
    """A compact version of the pins of tests/test_oracle_*.py; raises AssertionError on the first failure."""
    wl, rp, ci, X, home = workload
    cfg = wl.cfg
    # Philox known answers and the draw's block / word mapping
    assert [int(x) for x in orc.philox4x32_10([0] * 4, [0] * 2)] == [0x6627E8D5, 0xE169C58D, 0xBC57AC4C, 0x9B00DBD8]
    assert [int(x) for x in orc.philox4x32_10([0x243F6A88, 0x85A308D3, 0x13198A2E, 0x03707344], [0xA4093822, 0x299F31D0])] == \
        [0xD16CFE09, 0x94FDCCEB, 0x5001E420, 0x24126EA1]
    seed = 0x0123456789ABCDEF
    for i in range(9):
        blk = orc.philox4x32_10([77, 2, i >> 2, 5], [seed & 0xFFFFFFFF, seed >> 32])
        assert orc.draw(seed, 5, 77, 2, i) == int(blk[i & 3])
    # Floyd: golden vectors, whole rows, uniform subsets
    assert orc.sample_positions(42, 1, 7, 0, 100, 10).tolist() == [77, 76, 12, 90, 54, 20, 29, 70, 10, 46]
    assert orc.sample_positions(1, 0, 5, 0, 6, 5).tolist() == [0, 2, 3, 1, 5]
    assert orc.sample_positions(1, 0, 5, 0, 5, 5).tolist() == [0, 1, 2, 3, 4]
    subsets = Counter()
    for e in range(12_000):
        pos = orc.sample_positions(9, e, 3, 1, 5, 2)
        assert len(set(pos.tolist())) == 2 and 0 <= pos.min() and pos.max() < 5
        subsets[tuple(sorted(pos.tolist()))] += 1
    assert set(subsets) == set(itertools.combinations(range(5), 2))
    assert all(abs(c - 1200) < 5 * np.sqrt(1200 * 0.9) for c in subsets.values())
    # schedule
    assert orc.epoch_schedule(np.arange(8), 42, 0).tolist() == [2, 1, 0, 7, 3, 5, 6, 4]
    assert orc.epoch_schedule(np.arange(8), 42, 1).tolist() == [3, 1, 7, 0, 6, 5, 2, 4]
    # blocks: edges are real, counts, hop streams, dedup, relabelling
    seeds = orc.epoch_batches(wl.train_ids.numpy(), 64, wl.seed, 0)[0]
    b = orc.sample_blocks(rp, ci, seeds, (6, 4), 11, 2)
    assert len(set(b.nodes.tolist())) == b.nodes.size
    rows = {}
    for h in range(2):
        n_h = int(b.tier_off[h + 1])
        tier = b.nodes[b.tier_off[h + 1]:b.tier_off[h + 2]]
        assert np.all(np.diff(tier) > 0)
        assert np.array_equal(b.nodes[:b.tier_off[h + 2]][b.nbr_local[h]], b.nbr[h])
        for i in range(n_h):
            v = int(b.nodes[i])
            got = b.nbr[h][b.indptr[h][i]:b.indptr[h][i + 1]]
            row = ci[rp[v]:rp[v + 1]]
            assert got.size == min((6, 4)[h], row.size) and set(got.tolist()) <= set(row.tolist())
            assert len(set(got.tolist())) == got.size
            if row.size <= (6, 4)[h]:
                assert got.tolist() == row.tolist()
            rows[(h, v)] = got.tolist()
    # the first positions drawn for a high-degree seed follow the hop's own stream
    v = int(max(seeds, key=lambda s: rp[s + 1] - rp[s]))
    d = int(rp[v + 1] - rp[v])
    assert d > 6
    for h, k in ((0, 6), (1, 4)):
        want = [int(ci[rp[v] + p]) for p in orc.sample_positions(11, 2, v, h, d, k)]
        assert rows[(h, v)] == want
    # first-seen node order: same tiers as sets, positions handed out in order of first mention
    f = orc.sample_blocks(rp, ci, seeds, (6, 4), 11, 2, orc.ORDER_FIRST_SEEN)
    assert f.tier_off.tolist() == b.tier_off.tolist()
    for h in range(2):
        lo, hi = int(f.tier_off[h + 1]), int(f.tier_off[h + 2])
        assert sorted(f.nodes[lo:hi].tolist()) == b.nodes[lo:hi].tolist()
        assert np.array_equal(f.nodes[:hi][f.nbr_local[h]], f.nbr[h])
        next_free = lo
        for p in f.nbr_local[h].tolist():
            if p >= next_free:
                assert p == next_free
                next_free += 1
        assert next_free == hi
    # histogram, TopHot, fill, gather, hit curve
    counts = np.zeros(cfg.num_nodes, dtype=np.uint32)
    inputs = []
    for s in orc.epoch_batches(wl.train_ids.numpy(), cfg.batch_size, wl.seed, 0, 4):
        blk = orc.sample_blocks(rp, ci, s, cfg.fanouts, wl.seed, 0)
        orc.access_histogram(blk.input_nodes, counts)
        inputs.append(blk.input_nodes)
    assert np.array_equal(counts, np.bincount(np.concatenate(inputs), minlength=cfg.num_nodes).astype(np.uint32))
    ids, loc = orc.build_cache(counts, home, 300)
    tag = (home.astype(np.int64) & 0xFFFFFFFF) >> 30
    cand = np.flatnonzero((tag == 2) & (counts >= 1))
    order = cand[np.lexsort((cand, -counts[cand].astype(np.int64)))]
    assert ids.tolist() == np.sort(order[:300]).tolist()
    assert orc.build_cache(counts, home, 10 ** 6)[0].tolist() == cand.tolist()      # never a node nobody asked for
    assert np.array_equal(orc.fill_cache(X, ids), X[ids])
    hits = 0
    for nodes in inputs:
        out, st = orc.gather_features(X, nodes, loc)
        assert np.array_equal(out, X[nodes])
        t = (loc.astype(np.int64)[nodes] & 0xFFFFFFFF) >> 30
        assert st == tuple(int((t == x).sum()) for x in (0, 1, 2))
        hits += st[1]
    assert hits == int(counts[ids].sum())
    curve, total = orc.cache_hit_curve(counts, home, [0, 300, 10 ** 6])
    assert curve.tolist() == [0, hits, int(counts[cand].sum())] and total == int(counts[cand].sum())
    # mean aggregation
    agg = orc.mean_aggregate(np.array([0, 2, 2, 5]), np.array([1, 2, 3, 3, 4], dtype=np.int32), X[:8])
    assert np.allclose(agg[0], (X[1].astype(np.float64) + X[2]) / 2) and not agg[1].any()
    assert np.allclose(agg[2], (2 * X[3].astype(np.float64) + X[4]) / 3)


def test_unmodified_oracle_passes_the_compact_pins(tmp_path, workload):
    lib = _Lib(_build(str(tmp_path), "original"))
    try:
        _compact_pins(lib.mod, workload)
    finally:
        lib.close()


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, workload, name, old, new):
    lib = _Lib(_build(str(tmp_path), name, old, new))
    try:
        with pytest.raises(AssertionError):
            _compact_pins(lib.mod, workload)
    finally:
        lib.close()
