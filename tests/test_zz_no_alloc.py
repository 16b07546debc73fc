"""rg_gather_features_static (the entry point for callers that cannot allocate) against rg_gather_features.

Two calls in a row through the C ABI, the second with a smaller input: rows and statistics must equal those
of the allocating entry point bit for bit (and the oracle's), the device's free memory must not change across
the calls, and a row count beyond the static scratch is refused without queuing anything.
"""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_common import host_graph, log

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _sampled_batches(B, ctx, wl, n_batches):
    cfg, H = wl.cfg, len(wl.cfg.fanouts)
    csr = B.CsrGraph(wl.row_ptr, wl.col_idx)
    order = ctx.epoch_schedule(wl.train_ids, wl.seed, 0)
    counts = torch.zeros(cfg.num_nodes, dtype=torch.int32, device=DEV)
    nodes = []
    for b in range(n_batches):
        bufs = B.BlockBuffers(cfg.num_nodes, wl.nnz, cfg.batch_size, cfg.fanouts, DEV)
        seeds = order[b * cfg.batch_size:(b + 1) * cfg.batch_size]
        ctx.sample_blocks(csr, seeds, seeds.numel(), cfg.fanouts, wl.seed, 0, bufs)
        torch.cuda.synchronize()
        n = int(bufs.tier_off[H + 1].item())
        ctx.access_histogram(bufs.nodes, n, counts)
        nodes.append(bufs.nodes[:n].clone())
    return nodes, counts


@pytest.mark.parametrize("name,two_streams", [("small", True), ("tiny", False)])
def test_static_gather_matches_allocating_gather(name, two_streams):
    from paper_2505_10806_amd import binding as B
    log(f"[no-alloc] workload {name}, two_streams={two_streams}")
    wl = synth.build_workload(name, seed=11, device=DEV)
    cfg = wl.cfg
    ctx = B.Context(0)
    nodes, counts = _sampled_batches(B, ctx, wl, 2)
    cache = B.FeatureCache(cfg.num_nodes, min(wl.capacity_rows, wl.n_remote), wl.stride, DEV)
    ctx.build_cache(counts, wl.home, wl.remote_store, cfg.feat_dim, cache)
    torch.cuda.synchronize()
    X = wl.features.cpu().numpy()
    loc_np = cache.loc.cpu().numpy()
    side = torch.cuda.Stream() if two_streams else None

    n0 = nodes[0].numel()
    n1 = max(1, nodes[1].numel() // 7)                    # the second call is smaller than the first
    assert n1 < n0 <= B.RG_STATIC_GATHER_MAX_ROWS
    cap = max(n0, n1)
    want_out = torch.empty(cap, wl.stride, device=DEV)
    got_out = torch.empty(cap, wl.stride, device=DEV)
    want_st = torch.zeros(3, dtype=torch.int64, device=DEV)
    got_st = torch.zeros(3, dtype=torch.int64, device=DEV)
    n_dev = torch.zeros(1, dtype=torch.int32, device=DEV)

    # the allocating entry point first, so that its scratch growth is not charged to the calls under test
    refs = []
    for ids, n in ((nodes[0], n0), (nodes[1], n1)):
        want_out.fill_(-7.0)
        ctx.gather_features(ids, n, cache, wl.local_store, wl.remote_store, cfg.feat_dim, want_out, want_st, miss_stream=side)
        torch.cuda.synchronize()
        refs.append((want_out[:n].clone(), tuple(want_st.cpu().tolist())))

    for call, (ids, n) in enumerate(((nodes[0], n0), (nodes[1], n1))):
        log(f"[no-alloc] call {call}: n = {n}")
        got_out.fill_(-7.0)
        got_st.fill_(123)                                 # stale statistics must be overwritten, not accumulated
        torch.cuda.synchronize()
        free_before, _ = torch.cuda.mem_get_info()        # the driver's own figure, not the torch allocator's
        ctx.gather_features_static(ids, n, cache, wl.local_store, wl.remote_store, cfg.feat_dim, got_out, got_st,
                                   miss_stream=side)
        torch.cuda.synchronize()
        free_after, _ = torch.cuda.mem_get_info()
        assert free_after == free_before, "the device's free memory changed across the static call"
        ref_rows, ref_st = refs[call]
        assert tuple(got_st.cpu().tolist()) == ref_st
        assert torch.equal(got_out[:n], ref_rows), f"rows of call {call} differ from rg_gather_features"
        assert bool((got_out[n:] == -7.0).all()), "rows beyond n were written"
        want, st_orc = oracle.gather_features(X, ids[:n].cpu().numpy(), loc_np)
        assert ref_st == st_orc
        assert np.array_equal(got_out[:n, :cfg.feat_dim].cpu().numpy(), want)

    # a device-side count below n, and an empty call
    n_dev.fill_(5)
    got_out.fill_(-7.0)
    ctx.gather_features_static(nodes[0], n0, cache, wl.local_store, wl.remote_store, cfg.feat_dim, got_out, got_st,
                               n_dev=n_dev, miss_stream=side)
    torch.cuda.synchronize()
    assert int(got_st.sum().item()) == 5 and torch.equal(got_out[:5], refs[0][0][:5]) and bool((got_out[5:] == -7.0).all())
    ctx.gather_features_static(nodes[0], 0, cache, wl.local_store, wl.remote_store, cfg.feat_dim, got_out, got_st)
    torch.cuda.synchronize()
    assert got_st.cpu().tolist() == [0, 0, 0]

    # beyond the static scratch: refused on the host, nothing queued, the context keeps working
    big = torch.zeros(B.RG_STATIC_GATHER_MAX_ROWS + 1, dtype=torch.int32, device=DEV)
    big_out = torch.empty(1, wl.stride, device=DEV)       # never written: the call is refused before any launch
    with pytest.raises(B.RgError) as e:
        ctx.gather_features_static(big, big.numel(), cache, wl.local_store, wl.remote_store, cfg.feat_dim, big_out, got_st)
    assert e.value.status == B.RG_ERR_CAPACITY and "static scratch" in str(e.value)
    ctx.gather_features_static(nodes[1], n1, cache, wl.local_store, wl.remote_store, cfg.feat_dim, got_out, got_st)
    torch.cuda.synchronize()
    assert tuple(got_st.cpu().tolist()) == refs[1][1] and torch.equal(got_out[:n1], refs[1][0])
    ctx.close()


def test_static_gather_replays_from_a_hip_graph():
    """What the entry point is for: the call is captured into a HIP graph (nothing in it allocates, and its scratch sits at
    a fixed address) and replayed for new inputs written into the same buffers.  Each of three replays, with eager work
    and synchronisations between them, must give the rows and statistics of the eager call on the same input."""
    from paper_2505_10806_amd import binding as B
    wl = synth.build_workload("tiny", seed=13, device=DEV)
    cfg = wl.cfg
    ctx = B.Context(0)
    nodes, counts = _sampled_batches(B, ctx, wl, 3)
    cache = B.FeatureCache(cfg.num_nodes, min(wl.capacity_rows, wl.n_remote), wl.stride, DEV)
    ctx.build_cache(counts, wl.home, wl.remote_store, cfg.feat_dim, cache)
    cap = max(x.numel() for x in nodes)
    ids_buf = torch.zeros(cap, dtype=torch.int32, device=DEV)      # the graph reads its input here ...
    n_dev = torch.zeros(1, dtype=torch.int32, device=DEV)          # ... and the row count here
    out = torch.empty(cap, wl.stride, device=DEV)
    stats = torch.zeros(3, dtype=torch.int64, device=DEV)
    eager_out = torch.empty(cap, wl.stride, device=DEV)
    eager_stats = torch.zeros(3, dtype=torch.int64, device=DEV)

    def load(ids):
        ids_buf[:ids.numel()].copy_(ids)
        n_dev.fill_(ids.numel())

    load(nodes[0])
    ctx.gather_features_static(ids_buf, cap, cache, wl.local_store, wl.remote_store, cfg.feat_dim, out, stats, n_dev=n_dev)   # warm-up
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph.capture_begin(capture_error_mode="relaxed")
        ctx.gather_features_static(ids_buf, cap, cache, wl.local_store, wl.remote_store, cfg.feat_dim, out, stats, n_dev=n_dev)
        graph.capture_end()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for replay, ids in enumerate((nodes[1], nodes[2], nodes[0])):
        n = ids.numel()
        log(f"[no-alloc] graph replay {replay}: n = {n}")
        eager_out.fill_(-7.0)
        ctx.gather_features(ids, n, cache, wl.local_store, wl.remote_store, cfg.feat_dim, eager_out, eager_stats)   # eager work between replays
        torch.cuda.synchronize()
        load(ids)
        out.fill_(-7.0)
        stats.fill_(99)
        graph.replay()
        torch.cuda.synchronize()
        assert tuple(stats.cpu().tolist()) == tuple(eager_stats.cpu().tolist())
        assert torch.equal(out[:n], eager_out[:n]) and bool((out[n:] == -7.0).all())
    del graph
    ctx.close()
