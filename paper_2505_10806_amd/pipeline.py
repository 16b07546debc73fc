"""Epoch driver over the C-ABI binding: the offline stage of Alg. 1 (lines 1-4: precompute the
batches, count accesses, TopHot, VectorPull) followed by the online per-batch feature assembly
(lines 12-14).  Host code only sequences library calls and owns the buffers; every step runs in the
library's kernels.  No host synchronisation happens inside the offline stage: frontier sizes stay
on the device and are read back once, before the online stage.
"""
import torch

from . import binding as B


class EpochPipeline:
    def __init__(self, wl, device="cuda:0", max_batches=None, ctx=None, two_streams=True, prefetch=True,
                 epoch_histogram=True, sampler_streams=3):
        cfg = wl.cfg
        self.wl, self.cfg, self.device = wl, cfg, device
        self.H = len(cfg.fanouts)
        self.ctx = ctx or B.Context(torch.device(device).index or 0)
        self.csr = B.CsrGraph(wl.row_ptr, wl.col_idx)
        self.batches_per_epoch = wl.batches_per_epoch()
        self.max_batches = min(max_batches or self.batches_per_epoch, self.batches_per_epoch)
        # Batches are independent, and most sampler kernels of one batch are far smaller than the GPU: several
        # batches are sampled side by side, each lane with its own stream, context (scratch) and hop buffers.
        n_lanes = max(1, int(sampler_streams)) if epoch_histogram else 1
        self.lane_ctx = [self.ctx] + [B.Context(self.ctx.device) for _ in range(n_lanes - 1)]
        self.lane_bufs = [B.BlockBuffers(cfg.num_nodes, wl.nnz, cfg.batch_size, cfg.fanouts, device) for _ in range(n_lanes)]
        self.n_lanes = n_lanes
        self.bufs = self.lane_bufs[0]
        self.slot = self.bufs.frontier_ub[self.H]
        # one slot of input nodes and one row of tier offsets per precomputed batch
        self.arena = torch.empty(self.max_batches, max(self.slot, 1), dtype=torch.int32, device=device)
        self.tier_offs = torch.zeros(self.max_batches, self.H + 2, dtype=torch.int32, device=device)
        self.counts = torch.zeros(cfg.num_nodes, dtype=torch.int32, device=device)
        self.cache = B.FeatureCache(cfg.num_nodes, min(wl.capacity_rows, wl.n_remote), wl.stride, device)
        self.out = torch.empty(max(self.slot, 1), wl.stride, dtype=torch.float32, device=device)
        self.stats = torch.zeros(self.max_batches, 3, dtype=torch.int64, device=device)
        self.order = torch.empty_like(wl.train_ids)
        self.side = torch.cuda.Stream(device=device) if two_streams else None
        # prefetch = pull cached rows batch by batch, in order of first use, on a stream of their own so the
        # host-link transfer overlaps the gathers; otherwise one bulk pull right after TopHot
        self.prefetch = prefetch
        # one LDS-privatised histogram over the whole epoch instead of one global-atomic pass per batch
        self.epoch_histogram = epoch_histogram
        self.pf_stream = torch.cuda.Stream(device=device) if prefetch else None
        self.pf_events = [torch.cuda.Event() for _ in range(self.max_batches)] if prefetch else None
        # The sampler lanes reuse the streams that are idle during the offline stage (miss and prefetch streams);
        # only lanes beyond those get streams of their own.  The device exposes few hardware queues, and streams
        # that end up sharing one would serialise work that is meant to overlap.
        spare = [st for st in (self.side, self.pf_stream) if st is not None]
        self.lane_stream = [None] + spare[:self.n_lanes - 1]
        while len(self.lane_stream) < self.n_lanes:
            self.lane_stream.append(torch.cuda.Stream(device=device))
        for c in self.lane_ctx:
            c.reserve(cfg.num_nodes, self.slot, self.slot if c is self.ctx else 0)
        self.sizes = None

    # kernel timing over every lane's context
    def profile_enable(self, on=True):
        for c in self.lane_ctx:
            c.profile_enable(on)

    def profile_reset(self):
        for c in self.lane_ctx:
            c.profile_reset()

    def profile_read(self, kernel_id):
        ms, launches = 0.0, 0
        for c in self.lane_ctx:
            m, n = c.profile_read(kernel_id)
            ms, launches = ms + m, launches + n
        return ms, launches

    def precompute(self, epoch, n_batches=None, batch_ids=None):
        """Offline stage (asynchronous) for the first n_batches batches of `epoch`, or for the listed
        batch indices; slot i of the arena holds the i-th of them."""
        cfg, ctx = self.cfg, self.ctx
        ids = list(batch_ids) if batch_ids is not None else list(range(n_batches))
        assert len(ids) <= self.max_batches and all(0 <= b < self.batches_per_epoch for b in ids)
        ctx.epoch_schedule(self.wl.train_ids, self.wl.seed, epoch, self.order)
        self.counts.zero_()
        n_train = self.order.numel()
        main = torch.cuda.current_stream()
        lanes = len(self.lane_ctx)
        for st in self.lane_stream[1:]:
            st.wait_stream(main)
        for i, b in enumerate(ids):
            seeds = self.order[b * cfg.batch_size:min((b + 1) * cfg.batch_size, n_train)]
            lane = i % lanes
            bufs = self.lane_bufs[lane]
            bufs.set_outputs(self.arena[i], self.tier_offs[i])
            self.lane_ctx[lane].sample_blocks(self.csr, seeds, seeds.numel(), cfg.fanouts, self.wl.seed, epoch, bufs,
                                              stream=self.lane_stream[lane])
            if not self.epoch_histogram:
                ctx.access_histogram(self.arena[i], self.slot, self.counts, n_dev=self.tier_offs[i, self.H + 1:])
        for st in self.lane_stream[1:]:
            main.wait_stream(st)
        if self.epoch_histogram:
            ctx.access_histogram_epoch(self.arena, self.tier_offs, len(ids), self.H, cfg.batch_size, self.counts)
        ctx.build_cache(self.counts, self.wl.home, None if self.prefetch else self.wl.remote_store, cfg.feat_dim, self.cache)
        self.n_batches = len(ids)

    def read_sizes(self):
        """One device-to-host copy of every batch's tier offsets (synchronises)."""
        self.sizes = self.tier_offs[:self.n_batches, self.H + 1].cpu().tolist()
        return self.sizes

    def gather(self, b):
        """Online stage for batch b: features of its input nodes into self.out[:n]."""
        n = self.sizes[b]
        self.ctx.gather_features(self.arena[b], n, self.cache, self.wl.local_store, self.wl.remote_store,
                                 self.cfg.feat_dim, self.out, self.stats[b], miss_stream=self.side)
        return n

    def prefetch_rows(self, b, stream=None):
        """Pull the not-yet-resident cached rows batch b needs (asynchronous on `stream`)."""
        self.ctx.prefetch_cache_rows(self.arena[b], self.sizes[b], self.cache, self.wl.home, self.wl.remote_store,
                                     self.cfg.feat_dim, stream=stream)

    def online(self, n_batches):
        """Online stage: gathers in batch order; with prefetch on, batch b's gather waits only for the pulls
        of batches 0..b, which run ahead on the prefetch stream."""
        if not self.prefetch:
            for b in range(n_batches):
                self.gather(b)
            return
        main = torch.cuda.current_stream()
        self.pf_stream.wait_stream(main)
        for b in range(n_batches):
            self.prefetch_rows(b, stream=self.pf_stream)
            self.pf_events[b].record(self.pf_stream)
            main.wait_event(self.pf_events[b])
            self.gather(b)

    def run_epoch(self, epoch, n_batches):
        self.precompute(epoch, n_batches)
        self.read_sizes()
        self.online(n_batches)
