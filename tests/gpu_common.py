"""Helpers for the GPU parity tests: run the HIP path through the C-ABI binding and the oracle on the
same seeded inputs.  Nothing here computes expected values: those come from `oracle` only."""
import sys

import numpy as np
import torch

import oracle
import synth


def log(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def np_i64(t):
    return t.detach().cpu().numpy().astype(np.int64)


class HipBatch:
    """Host copies of one sampled batch produced by the HIP path."""

    def __init__(self, bufs, num_hops):
        torch.cuda.synchronize()
        self.tier_off = np_i64(bufs.tier_off)
        n = int(self.tier_off[num_hops + 1])
        self.nodes = bufs.nodes[:n].cpu().numpy()
        self.indptr, self.nbr, self.nbr_local = [], [], []
        for h in range(num_hops):
            n_h = int(self.tier_off[h + 1])
            ip = bufs.indptr[h][:n_h + 1].cpu().numpy()
            e = int(ip[-1])
            self.indptr.append(ip)
            self.nbr.append(bufs.nbr[h][:e].cpu().numpy())
            self.nbr_local.append(bufs.nbr_local[h][:e].cpu().numpy() if bufs.nbr_local else None)
        self.num_edges = bufs.num_edges.cpu().numpy().astype(np.int64)


def assert_batch_equal(hip, orc, num_hops, tag=""):
    assert hip.tier_off.tolist() == orc.tier_off.tolist(), f"{tag} tier_off"
    assert np.array_equal(hip.nodes, orc.nodes), f"{tag} nodes"
    assert hip.num_edges[:num_hops].tolist() == [int(x.size) for x in orc.nbr], f"{tag} num_edges"
    for h in range(num_hops):
        assert np.array_equal(hip.indptr[h].astype(np.int64), orc.indptr[h]), f"{tag} indptr[{h}]"
        assert np.array_equal(hip.nbr[h], orc.nbr[h]), f"{tag} nbr[{h}]"
        if hip.nbr_local[h] is not None:
            assert np.array_equal(hip.nbr_local[h], orc.nbr_local[h]), f"{tag} nbr_local[{h}]"


def host_graph(wl):
    return wl.row_ptr.cpu().numpy().astype(np.int64), wl.col_idx.cpu().numpy()


class OracleAhead:
    """Runs fn(item) for a list of items on a few host threads, a bounded number of items ahead of the
    consumer (the oracle is single-threaded C called through ctypes, which releases the GIL).  Results are
    handed out strictly in order; nothing about a result depends on the threading."""

    def __init__(self, fn, items, workers=8, window=12):
        import concurrent.futures
        self._pool = concurrent.futures.ThreadPoolExecutor(max_workers=workers)
        self._fn, self._items, self._window = fn, list(items), window
        self._futures, self._next_submit, self._next_take = {}, 0, 0
        self._fill()

    def _fill(self):
        while self._next_submit < len(self._items) and self._next_submit < self._next_take + self._window:
            self._futures[self._next_submit] = self._pool.submit(self._fn, self._items[self._next_submit])
            self._next_submit += 1

    def take(self):
        """Result for the next item (blocks until it is ready)."""
        i = self._next_take
        res = self._futures.pop(i).result()
        self._next_take += 1
        self._fill()
        return res

    def close(self):
        self._pool.shutdown(wait=True, cancel_futures=True)
