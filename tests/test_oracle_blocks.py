"""Pins for the oracle's multi-hop block sampler on tiny graphs (CPU only)."""
import numpy as np
import pytest
import scipy.sparse as sp
from scipy.sparse.csgraph import shortest_path

import oracle
import synth


@pytest.fixture(scope="module")
def tiny_graph():
    row_ptr, col_idx = synth.chung_lu_csr(2000, 12, 2.1, seed=3)
    return row_ptr.numpy().astype(np.int64), col_idx.numpy()


def _degree(rp, v):
    return int(rp[v + 1] - rp[v])


def _row(rp, ci, v):
    return ci[rp[v]:rp[v + 1]]


def test_synth_graph_is_symmetric_simple_sorted(tiny_graph):
    rp, ci = tiny_graph
    n = rp.size - 1
    a = sp.csr_matrix((np.ones(ci.size, dtype=np.int8), ci, rp), shape=(n, n))
    assert (a != a.T).nnz == 0
    assert a.diagonal().sum() == 0
    for v in range(n):
        r = _row(rp, ci, v)
        assert np.all(np.diff(r) > 0)       # sorted and duplicate free
    deg = np.diff(rp)
    assert deg.max() > 8 * deg.mean()       # heavy tail


@pytest.mark.parametrize("fanouts", [(10, 5), (3, 3, 3), (25,), (0, 4)])
def test_block_invariants(tiny_graph, fanouts):
    rp, ci = tiny_graph
    n = rp.size - 1
    rng = np.random.default_rng(5)
    seeds = rng.choice(n, size=64, replace=False).astype(np.int32)
    b = oracle.sample_blocks(rp, ci, seeds, fanouts, seed=11, epoch=2)
    H = len(fanouts)
    assert b.tier_off[0] == 0 and b.tier_off[1] == seeds.size
    assert b.nodes[:seeds.size].tolist() == seeds.tolist()
    assert len(set(b.nodes.tolist())) == b.nodes.size           # all ids unique
    for h in range(H):
        n_h = int(b.tier_off[h + 1])
        tier = b.nodes[b.tier_off[h + 1]:b.tier_off[h + 2]]
        assert np.all(np.diff(tier) > 0)                        # tier strictly ascending
        ip, nbr, loc = b.indptr[h], b.nbr[h], b.nbr_local[h]
        assert ip[0] == 0 and ip[-1] == nbr.size and ip.size == n_h + 1
        frontier_next = b.nodes[:b.tier_off[h + 2]]
        assert np.array_equal(frontier_next[loc], nbr)          # relabelling is consistent
        seen_new = set()
        for i in range(n_h):
            v = int(b.nodes[i])
            got = nbr[ip[i]:ip[i + 1]]
            d = _degree(rp, v)
            assert got.size == min(fanouts[h], d)               # (b) count = min(fanout, degree)
            row = set(_row(rp, ci, v).tolist())
            assert set(got.tolist()) <= row                      # (a) every neighbour is an edge
            assert len(set(got.tolist())) == got.size           # without replacement
            if d <= fanouts[h]:
                assert got.tolist() == _row(rp, ci, v).tolist()  # whole row, CSR order
            seen_new |= set(got.tolist())
        assert set(tier.tolist()) == seen_new - set(b.nodes[:n_h].tolist())


def test_rerun_and_batch_composition_independence(tiny_graph):
    rp, ci = tiny_graph
    n = rp.size - 1
    rng = np.random.default_rng(6)
    s1 = rng.choice(n, size=40, replace=False).astype(np.int32)
    s2 = np.concatenate([s1[:10][::-1], rng.choice(np.setdiff1d(np.arange(n), s1), 30, replace=False)]).astype(np.int32)
    a = oracle.sample_blocks(rp, ci, s1, (6, 4), seed=9, epoch=1)
    a2 = oracle.sample_blocks(rp, ci, s1, (6, 4), seed=9, epoch=1)
    assert a.nodes.tolist() == a2.nodes.tolist()                # (c) identical across reruns
    for h in range(2):
        assert a.nbr[h].tolist() == a2.nbr[h].tolist()
    b = oracle.sample_blocks(rp, ci, s2, (6, 4), seed=9, epoch=1)

    def rows(blk, h):
        n_h = int(blk.tier_off[h + 1])
        return {int(blk.nodes[i]): blk.nbr[h][blk.indptr[h][i]:blk.indptr[h][i + 1]].tolist() for i in range(n_h)}
    for h in range(2):
        ra, rb = rows(a, h), rows(b, h)
        common = set(ra) & set(rb)
        assert len(common) >= 10
        for v in common:                                         # the draw is keyed by node, not by batch
            assert ra[v] == rb[v]
    c = oracle.sample_blocks(rp, ci, s1, (6, 4), seed=9, epoch=2)
    d = oracle.sample_blocks(rp, ci, s1, (6, 4), seed=10, epoch=1)
    assert c.nbr[0].tolist() != a.nbr[0].tolist()               # different epoch -> different stream
    assert d.nbr[0].tolist() != a.nbr[0].tolist()               # different seed -> different stream
    assert rows(a, 0)[int(s1[0])] != rows(a, 1)[int(s1[0])] or _degree(rp, int(s1[0])) <= 4


@pytest.mark.parametrize("all_code", [-1, 10 ** 6])
def test_full_fanout_is_bfs_ball(tiny_graph, all_code):
    """With every fan-out >= the maximum degree the input nodes are the BFS ball of radius H:
    tier t holds exactly the nodes at distance t, ascending.  Checked against scipy's BFS."""
    rp, ci = tiny_graph
    n = rp.size - 1
    seeds = np.array([5, 900, 17], dtype=np.int32)
    H = 3
    b = oracle.sample_blocks(rp, ci, seeds, (all_code,) * H, seed=1, epoch=0)
    a = sp.csr_matrix((np.ones(ci.size), ci, rp), shape=(n, n))
    dist = shortest_path(a, method="D", unweighted=True, indices=seeds).min(axis=0)
    for t in range(1, H + 1):
        want = np.flatnonzero(dist == t)
        got = b.nodes[b.tier_off[t]:b.tier_off[t + 1]]
        assert got.tolist() == want.tolist()
    # each hop lists every edge of every frontier node
    for h in range(H):
        n_h = int(b.tier_off[h + 1])
        assert b.nbr[h].size == sum(_degree(rp, int(v)) for v in b.nodes[:n_h])


# ---- brute force: an independent, dictionary-and-bigint reimplementation on a hand-made graph

def _philox_py(ctr, key):
    c = list(ctr)
    k = list(key)
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def _blocks_py(adj, seeds, fanouts, seed, epoch, first_seen=False):
    key = (seed & 0xFFFFFFFF, seed >> 32)
    frontier = list(seeds)
    tiers, hops = [list(seeds)], []
    for h, k in enumerate(fanouts):
        rows = []
        for v in frontier:
            row = adj[v]
            d = len(row)
            if d <= k:
                chosen = list(range(d))
            else:
                chosen = []
                for i in range(k):
                    j = d - k + i
                    r = _philox_py((v, h, i >> 2, epoch), key)[i & 3]
                    t = (r * (j + 1)) >> 32
                    chosen.append(j if t in chosen else t)
            rows.append([row[c] for c in chosen])
        if first_seen:          # the order in which the hop's neighbour lists first name a node (dict keeps insertion order)
            new = list(dict.fromkeys(u for r in rows for u in r if u not in set(frontier)))
        else:
            new = sorted(set(u for r in rows for u in r) - set(frontier))
        frontier = frontier + new
        tiers.append(new)
        hops.append(rows)
    return frontier, tiers, hops


def test_blocks_against_bruteforce_python():
    rng = np.random.default_rng(8)
    n = 60
    adj = {v: [] for v in range(n)}
    for u in range(n):
        for v in range(u + 1, n):
            if rng.random() < (0.5 if u < 4 else 0.08):
                adj[u].append(v)
                adj[v].append(u)
    for v in adj:
        adj[v].sort()
    rp = np.zeros(n + 1, dtype=np.int64)
    rp[1:] = np.cumsum([len(adj[v]) for v in range(n)])
    ci = np.array([u for v in range(n) for u in adj[v]], dtype=np.int32)
    seeds = [7, 0, 33, 59]
    for fanouts, seed, epoch, first_seen in [((3, 2), 5, 0, False), ((5, 5, 1), (1 << 40) + 3, 9, False), ((2,), 0, 1, False),
                                             ((3, 2), 5, 0, True), ((5, 5, 1), (1 << 40) + 3, 9, True), ((4, 4, 4, 4), 7, 2, True)]:
        frontier, tiers, hops = _blocks_py(adj, seeds, fanouts, seed, epoch, first_seen)
        b = oracle.sample_blocks(rp, ci, seeds, fanouts, seed, epoch,
                                 oracle.ORDER_FIRST_SEEN if first_seen else oracle.ORDER_ASCENDING)
        assert b.nodes.tolist() == frontier
        for t, tier in enumerate(tiers):
            assert b.nodes[b.tier_off[t]:b.tier_off[t + 1]].tolist() == tier
        for h, rows in enumerate(hops):
            flat = [u for r in rows for u in r]
            assert b.nbr[h].tolist() == flat
            assert b.indptr[h].tolist() == np.concatenate([[0], np.cumsum([len(r) for r in rows])]).tolist()


def test_empty_and_isolated_inputs():
    rp = np.array([0, 0, 1, 2], dtype=np.int64)         # node 0 isolated, 1 <-> 2
    ci = np.array([2, 1], dtype=np.int32)
    b = oracle.sample_blocks(rp, ci, np.array([0], dtype=np.int32), (4, 4), 1, 0)
    assert b.nodes.tolist() == [0] and b.tier_off.tolist() == [0, 1, 1, 1]
    assert b.nbr[0].size == 0 and b.indptr[1].tolist() == [0, 0]
    e = oracle.sample_blocks(rp, ci, np.array([], dtype=np.int32), (4,), 1, 0)
    assert e.nodes.size == 0 and e.tier_off.tolist() == [0, 0, 0]
    c = oracle.sample_blocks(rp, ci, np.array([1], dtype=np.int32), (4, 4), 1, 0)
    assert c.nodes.tolist() == [1, 2] and c.nbr[1].tolist() == [2, 1] and c.nbr_local[1].tolist() == [1, 0]


# ---- randomised: the C oracle against the dictionary-and-bigint reimplementation on generated graphs
from hypothesis import HealthCheck, given, settings, strategies as st  # noqa: E402


@st.composite
def _graph_and_query(draw):
    n = draw(st.integers(2, 40))
    edges = draw(st.sets(st.tuples(st.integers(0, n - 1), st.integers(0, n - 1)), max_size=4 * n))
    adj = {v: set() for v in range(n)}
    for u, v in edges:
        if u != v:
            adj[u].add(v)
            adj[v].add(u)
    adj = {v: sorted(a) for v, a in adj.items()}
    seeds = draw(st.lists(st.integers(0, n - 1), min_size=0, max_size=min(n, 8), unique=True))
    fanouts = tuple(draw(st.lists(st.integers(0, 6), min_size=1, max_size=3)))
    seed = draw(st.integers(0, 2 ** 64 - 1))
    epoch = draw(st.integers(0, 2 ** 32 - 1))
    first_seen = draw(st.booleans())
    return n, adj, seeds, fanouts, seed, epoch, first_seen


@settings(max_examples=150, deadline=None, derandomize=True, suppress_health_check=list(HealthCheck))
@given(_graph_and_query())
def test_blocks_against_bruteforce_on_generated_graphs(case):
    n, adj, seeds, fanouts, seed, epoch, first_seen = case
    rp = np.zeros(n + 1, dtype=np.int64)
    rp[1:] = np.cumsum([len(adj[v]) for v in range(n)])
    ci = np.array([u for v in range(n) for u in adj[v]], dtype=np.int32)
    frontier, tiers, hops = _blocks_py(adj, seeds, fanouts, seed, epoch, first_seen)
    b = oracle.sample_blocks(rp, ci, np.array(seeds, dtype=np.int32), fanouts, seed, epoch,
                             oracle.ORDER_FIRST_SEEN if first_seen else oracle.ORDER_ASCENDING)
    assert b.nodes.tolist() == frontier
    assert b.tier_off.tolist() == np.concatenate([[0], np.cumsum([len(t) for t in tiers])]).tolist()
    for h, rows in enumerate(hops):
        assert b.nbr[h].tolist() == [u for r in rows for u in r]
        assert b.indptr[h].tolist() == np.concatenate([[0], np.cumsum([len(r) for r in rows])]).tolist()
        pos = {v: i for i, v in enumerate(b.nodes.tolist())}
        assert b.nbr_local[h].tolist() == [pos[u] for r in rows for u in r]


# ---- the second canonical node order: new nodes in the order in which the hop's neighbour list first names them

@pytest.mark.parametrize("fanouts", [(10, 5), (3, 3, 3), (25,), (0, 4)])
def test_first_seen_order_invariants(tiny_graph, fanouts):
    """Same tiers as sets and the same draw per node as the ascending order; inside a tier the nodes appear in the
    order of their first mention: walking nbr_local in edge order, every position beyond the old frontier that has
    not been met yet is exactly the next free position."""
    rp, ci = tiny_graph
    n = rp.size - 1
    rng = np.random.default_rng(15)
    seeds = rng.choice(n, size=64, replace=False).astype(np.int32)
    a = oracle.sample_blocks(rp, ci, seeds, fanouts, seed=11, epoch=2)
    f = oracle.sample_blocks(rp, ci, seeds, fanouts, seed=11, epoch=2, node_order=oracle.ORDER_FIRST_SEEN)
    H = len(fanouts)
    assert f.tier_off.tolist() == a.tier_off.tolist()
    assert f.nodes[:seeds.size].tolist() == seeds.tolist()
    assert len(set(f.nodes.tolist())) == f.nodes.size

    def rows(blk, h):
        n_h = int(blk.tier_off[h + 1])
        return {int(blk.nodes[i]): blk.nbr[h][blk.indptr[h][i]:blk.indptr[h][i + 1]].tolist() for i in range(n_h)}
    reordered = False
    for h in range(H):
        lo, hi = int(f.tier_off[h + 1]), int(f.tier_off[h + 2])
        tier_f, tier_a = f.nodes[lo:hi], a.nodes[lo:hi]
        assert sorted(tier_f.tolist()) == tier_a.tolist()                 # the same nodes, another order
        reordered = reordered or tier_f.tolist() != tier_a.tolist()
        assert rows(f, h) == rows(a, h)                                    # a node's draw does not depend on the order
        assert np.array_equal(f.nodes[:hi][f.nbr_local[h]], f.nbr[h])      # relabelling is consistent
        next_free = lo
        for p in f.nbr_local[h].tolist():
            if p >= next_free:
                assert p == next_free
                next_free += 1
        assert next_free == hi
    assert reordered or sum(fanouts) == 0


def test_first_seen_order_with_full_fanout_is_queue_bfs_order(tiny_graph):
    """Every neighbour taken, one seed: new nodes are discovered by scanning the frontier in order and each row in
    CSR order, which is the visiting order of a textbook queue BFS (scipy's breadth_first_order)."""
    from scipy.sparse.csgraph import breadth_first_order
    rp, ci = tiny_graph
    n = rp.size - 1
    a = sp.csr_matrix((np.ones(ci.size), ci, rp), shape=(n, n))
    for source in (5, 900):
        b = oracle.sample_blocks(rp, ci, np.array([source], dtype=np.int32), (-1, -1, -1), 1, 0, oracle.ORDER_FIRST_SEEN)
        order = breadth_first_order(a, source, directed=True, return_predecessors=False)
        assert b.nodes.size > 50
        assert b.nodes.tolist() == order[:b.nodes.size].tolist()
