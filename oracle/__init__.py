"""ctypes front end of the CPU oracle -- TEST INFRASTRUCTURE, not a product path.

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this package.  It never imports the HIP binding.  All arrays are numpy arrays in
host memory.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "librg_oracle.so")

TAG_LOCAL, TAG_CACHE, TAG_REMOTE = 0, 1, 2
TAG_SHIFT = 30


def build(force=False):
    """Compile rg_oracle.c with gcc into librg_oracle.so next to the source."""
    src = os.path.join(_HERE, "rg_oracle.c")
    hdr = os.path.join(_HERE, "rg_oracle.h")
    if (not force and os.path.exists(_LIB_PATH)
            and os.path.getmtime(_LIB_PATH) >= max(os.path.getmtime(src), os.path.getmtime(hdr))):
        return _LIB_PATH
    cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB_PATH, src]
    subprocess.run(cmd, check=True)
    return _LIB_PATH


_lib = None


def lib():
    global _lib
    if _lib is not None:
        return _lib
    build()
    L = ctypes.CDLL(_LIB_PATH)
    c_i64, c_i32, c_u64, c_u32 = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_uint32
    P = ctypes.c_void_p
    L.orc_philox4x32_10.argtypes = [P, P, P]
    L.orc_philox4x32_10.restype = None
    L.orc_draw.argtypes = [c_u64, c_u32, c_u32, c_u32, c_u64]
    L.orc_draw.restype = c_u32
    L.orc_sample_positions.argtypes = [c_u64, c_u32, c_u32, c_u32, c_i64, c_i64, P]
    L.orc_sample_positions.restype = c_i64
    L.orc_epoch_schedule.argtypes = [P, c_i64, c_u64, c_u32, P]
    L.orc_epoch_schedule.restype = None
    L.orc_sample_blocks.argtypes = [c_i64, P, P, P, c_i64, P, c_i32, c_u64, c_u32]
    L.orc_sample_blocks.restype = P
    L.orc_sample_blocks_ordered.argtypes = [c_i64, P, P, P, c_i64, P, c_i32, c_u64, c_u32, c_i32]
    L.orc_sample_blocks_ordered.restype = P
    L.orc_blocks_free.argtypes = [P]
    L.orc_blocks_free.restype = None
    L.orc_blocks_num_hops.argtypes = [P]
    L.orc_blocks_num_hops.restype = c_i32
    L.orc_blocks_tier_off.argtypes = [P]
    L.orc_blocks_tier_off.restype = ctypes.POINTER(c_i64)
    L.orc_blocks_nodes.argtypes = [P]
    L.orc_blocks_nodes.restype = ctypes.POINTER(c_i32)
    L.orc_blocks_num_edges.argtypes = [P, c_i32]
    L.orc_blocks_num_edges.restype = c_i64
    L.orc_blocks_indptr.argtypes = [P, c_i32]
    L.orc_blocks_indptr.restype = ctypes.POINTER(c_i64)
    L.orc_blocks_nbr.argtypes = [P, c_i32]
    L.orc_blocks_nbr.restype = ctypes.POINTER(c_i32)
    L.orc_blocks_nbr_local.argtypes = [P, c_i32]
    L.orc_blocks_nbr_local.restype = ctypes.POINTER(c_i32)
    L.orc_access_histogram.argtypes = [P, c_i64, P, c_i64]
    L.orc_access_histogram.restype = None
    L.orc_build_cache.argtypes = [P, P, c_i64, c_i64, P, P]
    L.orc_build_cache.restype = c_i64
    L.orc_fill_cache.argtypes = [P, c_i64, P, c_i64, P, c_i64]
    L.orc_fill_cache.restype = None
    L.orc_gather_features.argtypes = [P, c_i64, P, c_i64, P, P, c_i64, P]
    L.orc_gather_features.restype = None
    L.orc_cache_hit_curve.argtypes = [P, P, c_i64, P, c_i64, P]
    L.orc_cache_hit_curve.restype = c_u64
    L.orc_mean_aggregate.argtypes = [P, P, c_i64, P, c_i64, c_i64, P]
    L.orc_mean_aggregate.restype = None
    _lib = L
    return L


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _copy(ptr, n, dtype):
    if n == 0:
        return np.empty(0, dtype=dtype)
    return np.ctypeslib.as_array(ptr, shape=(n,)).astype(dtype, copy=True)


def philox4x32_10(ctr, key):
    c = _arr(ctr, np.uint32)
    k = _arr(key, np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def draw(seed, epoch, node, hop, i):
    return int(lib().orc_draw(seed, epoch, node, hop, i))


def sample_positions(seed, epoch, node, hop, d, k):
    m = d if (k < 0 or d <= k) else k
    pos = np.zeros(max(m, 1), dtype=np.int64)
    got = lib().orc_sample_positions(seed, epoch, node, hop, d, k, _p(pos))
    assert got == m
    return pos[:m].copy()


def epoch_schedule(train_ids, seed, epoch):
    t = _arr(train_ids, np.int32)
    out = np.empty_like(t)
    lib().orc_epoch_schedule(_p(t), t.size, seed, epoch, _p(out))
    return out


def epoch_batches(train_ids, batch_size, seed, epoch, max_batches=None):
    """The epoch order cut into consecutive batches; the partial last batch is kept."""
    order = epoch_schedule(train_ids, seed, epoch)
    out = [order[i:i + batch_size] for i in range(0, order.size, batch_size)]
    return out if max_batches is None else out[:max_batches]


class Blocks:
    """Result of sample_blocks: plain numpy arrays."""

    def __init__(self, tier_off, nodes, indptr, nbr, nbr_local):
        self.tier_off = tier_off      # int64 [H+2]
        self.nodes = nodes            # int32 [tier_off[-1]]
        self.indptr = indptr          # list of int64 [n_h+1]
        self.nbr = nbr                # list of int32 [E_h]
        self.nbr_local = nbr_local    # list of int32 [E_h]

    @property
    def input_nodes(self):
        return self.nodes


ORDER_ASCENDING, ORDER_FIRST_SEEN = 0, 1


def sample_blocks(row_ptr, col_idx, seeds, fanouts, seed, epoch, node_order=ORDER_ASCENDING):
    rp = _arr(row_ptr, np.int64)
    ci = _arr(col_idx, np.int32)
    sd = _arr(seeds, np.int32)
    fo = _arr(fanouts, np.int32)
    L = lib()
    h = L.orc_sample_blocks_ordered(rp.size - 1, _p(rp), _p(ci), _p(sd), sd.size, _p(fo), fo.size, seed, epoch, int(node_order))
    try:
        H = fo.size
        tier_off = _copy(L.orc_blocks_tier_off(h), H + 2, np.int64)
        nodes = _copy(L.orc_blocks_nodes(h), int(tier_off[-1]), np.int32)
        indptr, nbr, nbr_local = [], [], []
        for hop in range(H):
            e = L.orc_blocks_num_edges(h, hop)
            indptr.append(_copy(L.orc_blocks_indptr(h, hop), int(tier_off[hop + 1]) + 1, np.int64))
            nbr.append(_copy(L.orc_blocks_nbr(h, hop), e, np.int32))
            nbr_local.append(_copy(L.orc_blocks_nbr_local(h, hop), e, np.int32))
    finally:
        L.orc_blocks_free(h)
    return Blocks(tier_off, nodes, indptr, nbr, nbr_local)


def access_histogram(nodes, counts):
    """counts (uint32 [N], modified in place) += occurrences of each id in nodes."""
    nd = _arr(nodes, np.int32)
    assert counts.dtype == np.uint32 and counts.flags.c_contiguous
    lib().orc_access_histogram(_p(nd), nd.size, _p(counts), counts.size)
    return counts


def build_cache(counts, home, capacity_rows):
    """Returns (cache_ids int32 [K_eff] ascending, loc int32 [N])."""
    c = _arr(counts, np.uint32)
    hm = _arr(home, np.int32)
    ids = np.zeros(max(min(int(capacity_rows), c.size), 1), dtype=np.int32)
    loc = np.empty_like(hm)
    k = lib().orc_build_cache(_p(c), _p(hm), c.size, int(capacity_rows), _p(ids), _p(loc))
    return ids[:k].copy(), loc


def fill_cache(X, cache_ids, row_stride=None):
    X = _arr(X, np.float32)
    n, d = X.shape
    ids = _arr(cache_ids, np.int32)
    stride = d if row_stride is None else int(row_stride)
    rows = np.zeros((max(ids.size, 1), stride), dtype=np.float32)
    lib().orc_fill_cache(_p(X), d, _p(ids), ids.size, _p(rows), stride)
    return rows[:ids.size]


def gather_features(X, input_nodes, loc, out_stride=None):
    """Returns (out fp32 [n, out_stride], (n_local, n_hit, n_miss))."""
    X = _arr(X, np.float32)
    n_all, d = X.shape
    nd = _arr(input_nodes, np.int32)
    lc = _arr(loc, np.int32)
    stride = d if out_stride is None else int(out_stride)
    out = np.zeros((max(nd.size, 1), stride), dtype=np.float32)
    stats = np.zeros(3, dtype=np.int64)
    lib().orc_gather_features(_p(X), d, _p(nd), nd.size, _p(lc), _p(out), stride, _p(stats))
    return out[:nd.size], tuple(int(s) for s in stats)


def mean_aggregate(indptr, nbr_local, feat):
    """Mean of the source rows of every destination of a block, fp64 [n_dst, dim]; feat is fp32 [rows, dim]."""
    ip = _arr(indptr, np.int64)
    nl = _arr(nbr_local, np.int32)
    F = _arr(feat, np.float32)
    n_dst = ip.size - 1
    out = np.zeros((max(n_dst, 1), F.shape[1]), dtype=np.float64)
    lib().orc_mean_aggregate(_p(ip), _p(nl), n_dst, _p(F), F.shape[1], F.shape[1], _p(out))
    return out[:n_dst]


def cache_hit_curve(counts, home, capacities):
    """(hits uint64 [len(capacities)], total requests for remote rows)."""
    c = _arr(counts, np.uint32)
    hm = _arr(home, np.int32)
    caps = _arr(capacities, np.int64)
    hits = np.zeros(max(caps.size, 1), dtype=np.uint64)
    total = lib().orc_cache_hit_curve(_p(c), _p(hm), c.size, _p(caps), caps.size, _p(hits))
    return hits[:caps.size], int(total)
