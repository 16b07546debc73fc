"""Epoch driver over the C-ABI binding: the offline stage of Alg. 1 (lines 1-4: precompute the
batches, count accesses, TopHot, VectorPull) followed by the online per-batch feature assembly
(lines 12-14), with the paper's two latency-hiding devices mapped onto HIP streams:

* prefetcher (Section III, Fig. 4): cached rows are pulled over the host link batch by batch, in order of
  first use, on a stream of their own, one event per batch; gather b waits for event b only;
* double-buffered cache (Alg. 1 lines 7-8 and 18-20, C_s / C_sec): while epoch e is served, epoch e+1 is
  precomputed on another stream into the second buffer set, its rows are pulled behind epoch e's, and the
  buffers are swapped at the epoch boundary.

Further choices of the driver, each a constructor argument:

* a cache that can hold the whole remote partition is laid out as its mirror and filled while the batches are still
  being sampled, one pull per sampler call, its rows read off the sampler's membership bitmaps (mirror_cache,
  mirror_pulls, keep_rows);
* the pull stream can be bound to a few compute units of its own, every other stream to the rest (pull_cus; the
  caller then works on work_stream);
* when batches can have miss rows, their copies follow each other on the miss stream instead of being forked and
  joined per batch (decoupled_misses); when they cannot, the empty miss pass stays on the gather stream.

Host code only sequences library calls and owns the buffers; every step runs in the library's kernels.
No host synchronisation happens inside the offline stage: frontier sizes stay on the device.  They are
copied to pinned host memory as soon as the last batch has been sampled, so the host can size and queue the
online stage's launches while the histogram, TopHot and the prefetch plan are still running.
"""
import torch

from . import binding as B


class _EpochState:
    """Everything one precomputed epoch owns: input-node lists, tier offsets, counts and the cache."""

    def __init__(self, wl, H, slot, max_batches, device, keep_hops=None, mirror=False):
        cfg = wl.cfg
        # per-batch blocks that outlive the sampling call: hop -> (indptr, nbr, nbr_local), each [max_batches, cap].
        # The outermost hop is kept for the consumer of the gathered rows; all hops when every block is wanted.
        self.blk = {}
        for h, (n_ip, n_e) in (keep_hops or {}).items():
            self.blk[h] = tuple(torch.empty(max_batches, max(c, 1), dtype=torch.int32, device=device) for c in (n_ip, n_e, n_e))
        # one slot of input nodes and one row of tier offsets per precomputed batch
        self.arena = torch.empty(max_batches, max(slot, 1), dtype=torch.int32, device=device)
        self.tier_offs = torch.zeros(max_batches, H + 2, dtype=torch.int32, device=device)
        self.edge_counts = torch.zeros(max_batches, H, dtype=torch.int32, device=device)
        self.counts = torch.zeros(cfg.num_nodes, dtype=torch.int32, device=device)
        self.cache = B.FeatureCache(cfg.num_nodes, min(wl.capacity_rows, wl.n_remote), wl.stride, device,
                                    mirror_rows=wl.n_remote if mirror else 0, home=wl.home if mirror else None)
        self.stats = torch.zeros(max_batches, 3, dtype=torch.int64, device=device)
        self.pf_events = [torch.cuda.Event() for _ in range(max_batches)]
        self.sampled = [torch.cuda.Event() for _ in range(max_batches)]
        self.first_batch = None                # per node: first batch of the epoch that needs it (planned prefetch)
        self.plan = None
        self.built = torch.cuda.Event()        # offline stage of this state finished
        self.served = torch.cuda.Event()       # online stage of this state finished
        self.sizes = None
        self.sizes_host = torch.zeros(max_batches, H + 2, dtype=torch.int32).pin_memory()
        self.sizes_ready = torch.cuda.Event()  # the copy of the tier offsets into sizes_host has finished
        self.n_batches = 0
        self.pulls_queued = False


class EpochPipeline:
    def __init__(self, wl, device="cuda:0", max_batches=None, ctx=None, two_streams=True, prefetch=True,
                 histogram="epoch", sampler_streams=2, double_buffer=False,
                 queue_depth=1, consumer=None, planned_prefetch=True, sample_group=8, keep_blocks=False,
                 node_order="ascending", period_epochs=1, mirror_cache=None, keep_rows=False, mirror_pulls="group",
                 pull_cus=0, decoupled_misses=True):
        cfg = wl.cfg
        self.wl, self.cfg, self.device = wl, cfg, device
        self.H = len(cfg.fanouts)
        self._own_ctx = ctx is None
        self.ctx = ctx or B.Context(torch.device(device).index or 0)
        self.csr = B.CsrGraph(wl.row_ptr, wl.col_idx)
        self.batches_per_epoch = wl.batches_per_epoch()
        # period_epochs = E: the batches of E consecutive epochs are precomputed together, counted together and served
        # from one cache (Alg. 1 lines 1-4 as written: N, the frequencies and C_s cover every precomputed epoch); E = 1
        # builds a cache per epoch from that epoch's counts alone (the C_sec of Alg. 1 line 8).  A period's batches
        # occupy consecutive slots: epoch by epoch, batch by batch.
        self.period_epochs = max(1, int(period_epochs))
        self.max_batches = min(max_batches or self.batches_per_epoch, self.batches_per_epoch) * self.period_epochs
        # Batches are independent, and most sampler kernels of one batch are far smaller than the GPU: several
        # batches are sampled side by side, each lane with its own stream, context (scratch) and hop buffers.
        # node order inside a tier: "ascending" by id, or "first_seen" (the order in which the hop's neighbour list first
        # names a node).  Access counts: "epoch" = one LDS-privatised pass over all id lists after sampling (needs
        # ascending tiers), "sampled" = straight from the sampler's membership bitmaps after every group (any order, no
        # id list read), "batch" = one global-atomic pass per batch.
        if node_order not in ("ascending", "first_seen") or histogram not in ("epoch", "sampled", "batch"):
            raise ValueError("node_order must be 'ascending' or 'first_seen'; histogram 'epoch', 'sampled' or 'batch'")
        if node_order == "first_seen" and histogram == "epoch":
            histogram = "sampled"
        self.node_order = B.RG_ORDER_FIRST_SEEN if node_order == "first_seen" else B.RG_ORDER_ASCENDING
        self.histogram = histogram
        n_lanes = max(1, int(sampler_streams)) if histogram != "batch" else 1
        if double_buffer:
            n_lanes = max(n_lanes, 2)
        self.n_lanes = n_lanes
        self.lane_ctx = [self.ctx] + [B.Context(self.ctx.device) for _ in range(n_lanes - 1)]
        # every lane samples sample_group batches per call (one launch per kernel for the whole group)
        self.sample_group = max(1, min(int(sample_group), B.RG_MAX_GROUP))
        self.lane_bufs = [[B.BlockBuffers(cfg.num_nodes, wl.nnz, cfg.batch_size, cfg.fanouts, device)
                           for _ in range(self.sample_group)] for _ in range(n_lanes)]
        self.bufs = self.lane_bufs[0][0]
        self.slot = self.bufs.frontier_ub[self.H]
        self.double_buffer = double_buffer
        # consumer = "mean": the gathered rows of every batch are reduced by the mean aggregator over the batch's
        # outermost block (the first GraphSAGE layer's AGG) on a stream of its own; the gathers run up to
        # queue_depth batches ahead of it through a ring of output buffers (the paper's prefetch queue, Q = 3)
        if consumer not in (None, "mean"):
            raise ValueError("consumer must be None or 'mean'")
        self.consumer = consumer
        self.queue_depth = max(1, int(queue_depth))
        # decoupled misses: when batches can have miss rows, their copies over the host link run on the miss stream one
        # batch behind the other with nothing between them (forked once per group of lookups instead of once per batch,
        # joined per batch on the gather stream only), which needs a second output buffer to write ahead into
        self.decoupled = bool(decoupled_misses and two_streams and wl.capacity_rows < wl.n_remote)
        if self.decoupled:
            self.queue_depth = max(self.queue_depth, 2)
        # keep_blocks: every hop's block of every batch stays in per-batch buffers (the sampler writes them there
        # directly), e.g. to hand whole message-flow graphs to a trainer or to compare them after the epoch
        hops = range(self.H) if keep_blocks else ([self.H - 1] if consumer else [])
        keep = {h: (self.bufs.frontier_ub[h] + 1, self.bufs.edges_ub[h]) for h in hops}
        # When the cache can hold the whole remote partition, every remote row a batch names will be cached, so its
        # place can be fixed before TopHot has run: the cache is laid out as a mirror of the remote store and each
        # batch's rows are pulled as soon as the batch has been sampled, while the rest of the period is still being
        # sampled.  The host link then works through the offline stage instead of idling until TopHot is done.
        # keep_rows: rows pulled in an earlier period stay resident (features do not change), so later periods only
        # pull rows no period has named before; off = every period starts from a cold cache.
        self.no_misses = wl.capacity_rows >= wl.n_remote      # every remote row a period names is selected and pulled
        can_mirror = bool(prefetch and wl.n_remote > 0 and wl.capacity_rows >= wl.n_remote)
        self.mirror = can_mirror if mirror_cache is None else bool(mirror_cache and can_mirror)
        self.keep_rows = bool(keep_rows and self.mirror)
        # mirror_pulls: "group" = one pull per sampler call, its list read off the sampler's membership bitmaps (the
        # remote nodes the call's batches are the first of the period to name); "batch" = one pull per batch, each
        # preceded by a pass over the batch's id list that claims its not-yet-resident rows
        if mirror_pulls not in ("group", "batch"):
            raise ValueError("mirror_pulls must be 'group' or 'batch'")
        self.group_pulls = self.mirror and mirror_pulls == "group"
        self.states = [_EpochState(wl, self.H, self.slot, self.max_batches, device, keep, mirror=self.mirror)
                       for _ in range(2 if double_buffer else 1)]
        if self.keep_rows and len(self.states) > 1:
            # one physical mirror serves both buffer sets: the location tables, counts and cache ids are per period, the rows are not
            for st in self.states[1:]:
                st.cache = B.FeatureCache.sharing_rows(self.states[0].cache, cfg.num_nodes, device)
        if self.group_pulls:
            words = (cfg.num_nodes + 31) // 32
            for j, st in enumerate(self.states):
                st.plan = B.PrefetchPlan(wl.n_remote, self.max_batches, device)
                st.claimed = (self.states[0].claimed if self.keep_rows and j > 0 else
                              torch.zeros(words, dtype=torch.int32, device=device))
                st.claim_done = [torch.cuda.Event() for _ in range(self.max_batches)]
        self.cur = 0
        self.out_ring = [torch.empty(max(self.slot, 1), wl.stride, dtype=torch.float32, device=device)
                         for _ in range(self.queue_depth)]
        self.out = self.out_ring[0]                # the buffer the most recent gather wrote
        self.consumer_stream = torch.cuda.Stream(device=device) if consumer else None
        self.ready = [torch.cuda.Event() for _ in range(self.queue_depth)]
        self.consumed = [torch.cuda.Event() for _ in range(self.queue_depth)]
        self.rows_done = [torch.cuda.Event() for _ in range(self.queue_depth)]   # HBM-served half of the slot's batch copied
        self.miss_done = [torch.cuda.Event() for _ in range(self.queue_depth)]   # miss half copied
        self.prep_done = [torch.cuda.Event(), torch.cuda.Event()]                # lookups of a group made (one per half of the tickets)
        self._fork_due = {}                                                      # first ticket of a prepared group -> its half
        self.agg = (torch.empty(max(self.bufs.frontier_ub[self.H - 1], 1), wl.stride, dtype=torch.float32, device=device)
                    if consumer else None)
        self._gathered = 0
        self._tickets = {}                         # ticket -> (epoch state, batch) it is prepared for
        self.orders = [torch.empty_like(wl.train_ids) for _ in range(self.period_epochs)]
        self.order = self.orders[0]
        # pull_cus > 0: the prefetch stream gets that many compute units to itself and every other stream of the pipeline
        # (and self.work_stream, for the caller's gathers) the rest, so that no other kernel's wavefronts share a unit
        # with the few wavefronts that sit waiting on the host link
        self.pull_cus = int(pull_cus) if prefetch else 0
        n_cus = self.ctx.num_cus
        if self.pull_cus and not 0 < self.pull_cus < n_cus:
            raise ValueError("pull_cus must leave compute units for the other streams")
        def new_stream(role):
            if not self.pull_cus:
                return torch.cuda.Stream(device=device)
            # (process-wide streams, shared by all pipelines: torch objects may refer to a stream for longer than a pipeline lives)
            lo, n = (0, self.pull_cus) if role == "pulls" else (self.pull_cus, n_cus - self.pull_cus)
            return B.shared_stream_on_cus(self.ctx.device, lo, n, role)
        self.work_stream = new_stream("work") if self.pull_cus else None
        self.side = new_stream("side") if two_streams else None
        # prefetch = pull cached rows batch by batch, in order of first use, on a stream of their own so the
        # host-link transfer overlaps the gathers; otherwise one bulk pull right after TopHot
        self.prefetch = prefetch
        self.pf_stream = new_stream("pulls") if prefetch else None
        # planned prefetch: the epoch histogram also records the first batch that needs each node, the selected
        # slots are grouped by that batch once, and the prefetch stream then carries nothing but pulls
        self.planned = bool(prefetch and planned_prefetch and histogram != "batch" and not self.mirror)
        if self.planned:
            for st in self.states:
                st.first_batch = torch.empty(cfg.num_nodes, dtype=torch.int32, device=device)
                st.plan = B.PrefetchPlan(min(wl.capacity_rows, wl.n_remote), self.max_batches, device)
        # The sampler lanes reuse the streams that are idle during the offline stage (miss and prefetch streams);
        # only lanes beyond those get streams of their own.  The device exposes few hardware queues, and streams
        # that end up sharing one would serialise work that is meant to overlap.
        spare = [st for st in (self.side, None if self.mirror else self.pf_stream) if st is not None]
        self.lane_stream = [None] + spare[:self.n_lanes - 1]
        while len(self.lane_stream) < self.n_lanes:
            self.lane_stream.append(new_stream(("lane", len(self.lane_stream))))
        # with double buffering the next epoch is precomputed on one stream of its own while the current one is served
        self.build_stream = new_stream("build") if double_buffer else None
        for c in self.lane_ctx:
            c.reserve(cfg.num_nodes, self.slot, self.slot if c is self.ctx else 0, self.sample_group)

    def close(self):
        """Waits for the device and releases the sampler lanes' contexts.  The pipeline cannot be used afterwards."""
        torch.cuda.synchronize(self.device)
        for c in self.lane_ctx:
            if c is not self.ctx or self._own_ctx:       # a context the caller passed in stays the caller's
                c.close()

    # ---- the current epoch's buffers under their historical names
    @property
    def state(self):
        return self.states[self.cur]

    arena = property(lambda self: self.state.arena)
    tier_offs = property(lambda self: self.state.tier_offs)
    edge_counts = property(lambda self: self.state.edge_counts)
    counts = property(lambda self: self.state.counts)
    stats = property(lambda self: self.state.stats)
    sizes = property(lambda self: self.state.sizes)
    n_batches = property(lambda self: self.state.n_batches)

    @property
    def cache(self):
        return self.state.cache

    @cache.setter
    def cache(self, value):
        self.state.cache = value

    # ---- kernel timing over every lane's context
    def profile_enable(self, on=True):
        for c in self.lane_ctx:
            c.profile_enable(on)

    def profile_select(self, kernel_ids=None):
        for c in self.lane_ctx:
            c.profile_select(kernel_ids)

    def profile_reset(self):
        for c in self.lane_ctx:
            c.profile_reset()

    def profile_read(self, kernel_id):
        ms, launches = 0.0, 0
        for c in self.lane_ctx:
            m, n = c.profile_read(kernel_id)
            ms, launches = ms + m, launches + n
        return ms, launches

    # ---- offline stage
    def _offline(self, st, epoch, batch_ids, lanes):
        """Queue schedule, sampling, histogram and TopHot of one period (the listed batches of period_epochs epochs
        starting at `epoch`).  lanes = [(ctx, bufs, stream or None)]; lane 0's stream (None = the current stream) also
        runs the schedules, the histogram and TopHot."""
        cfg = self.cfg
        head_ctx, _, head_stream = lanes[0]
        head = head_stream or torch.cuda.current_stream()
        ids = [(k, b) for k in range(self.period_epochs) for b in batch_ids]          # slot -> (epoch of the period, batch)
        with torch.cuda.stream(head):
            for k in range(self.period_epochs):
                head_ctx.epoch_schedule(self.wl.train_ids, self.wl.seed, epoch + k, self.orders[k])
            st.counts.zero_()
            if self.planned:
                st.first_batch.fill_(-1)
            if self.mirror:
                if not self.keep_rows:
                    st.cache.filled.zero_()               # a cold cache: no row of the mirror is resident
                    if self.group_pulls:
                        st.claimed.zero_()
                if self.group_pulls:
                    st.plan.offsets[:1].zero_()
                self.pf_stream.wait_stream(head)
            for _, _, s in lanes[1:]:
                s.wait_stream(head)
            n_train = self.order.numel()
            gsz = self.sample_group
            if self.group_pulls:
                st.plan.set_num_batches(self.max_batches)
            # a sampling call takes batches of one epoch (the epoch is part of the draw's key)
            calls = []
            for k in range(self.period_epochs):
                i0 = k * len(batch_ids)
                for size in self._call_sizes(len(batch_ids), gsz, first=k == 0, last=k == self.period_epochs - 1):
                    calls.append((k, i0, i0 + size))
                    i0 += size
            for call, (k, i0, i1) in enumerate(calls):
                c, bufs_list, s = lanes[call % len(lanes)]
                seeds_list, outs = [], []
                for j, i in enumerate(range(i0, i1)):
                    b = ids[i][1]
                    seeds_list.append(self.orders[k][b * cfg.batch_size:min((b + 1) * cfg.batch_size, n_train)])
                    bufs = bufs_list[j]
                    bufs.set_outputs(st.arena[i], st.tier_offs[i], st.edge_counts[i])
                    for h, (ip, nb, nl) in st.blk.items():
                        bufs.set_hop(h, ip[i], nb[i], nl[i])
                    outs.append(bufs)
                c.sample_blocks_group(self.csr, seeds_list, cfg.fanouts, self.wl.seed, epoch + k, outs, stream=s or head,
                                      node_order=self.node_order)
                if self.histogram == "sampled":           # the group's membership bitmaps go straight into the counts
                    c.access_histogram_sampled(len(outs), st.counts, batch_index=range(i0, i0 + len(outs)),
                                               first_batch=st.first_batch, stream=s or head)
                if self.group_pulls:                      # this call's new remote rows start crossing the link now
                    if call > 0:                          # claims go in call order: each builds on the nodes claimed so far
                        (s or head).wait_event(st.claim_done[call - 1])
                    c.plan_sampled(len(outs), st.cache, st.claimed, st.plan, call, stream=s or head)
                    st.claim_done[call].record(s or head)
                    self.pf_stream.wait_event(st.claim_done[call])
                    self.ctx.prefetch_planned(st.plan, call, st.cache, self.wl.remote_store, cfg.feat_dim, stream=self.pf_stream)
                    for i in range(i0, i1):
                        st.pf_events[i].record(self.pf_stream)
                elif self.mirror:                         # each batch's not-yet-resident remote rows, batch by batch
                    st.sampled[i0].record(s or head)
                    self.pf_stream.wait_event(st.sampled[i0])
                    for i in range(i0, i1):
                        self.ctx.prefetch_cache_rows(st.arena[i], self.slot, st.cache, self.wl.home, self.wl.remote_store,
                                                     cfg.feat_dim, n_dev=st.tier_offs[i, self.H + 1:], stream=self.pf_stream)
                        st.pf_events[i].record(self.pf_stream)
                if self.histogram == "batch":
                    for i in range(i0, i1):
                        head_ctx.access_histogram(st.arena[i], self.slot, st.counts, n_dev=st.tier_offs[i, self.H + 1:], stream=head)
            for _, _, s in lanes[1:]:
                head.wait_stream(s)
            # the host needs the batch sizes to shape the online stage's launches: copy them out now, so that it can
            # queue that stage while the histogram, TopHot and the plan below are still running
            st.sizes_host[:len(ids)].copy_(st.tier_offs[:len(ids)], non_blocking=True)
            st.sizes_ready.record(head)
            if self.histogram == "epoch":
                head_ctx.access_histogram_epoch(st.arena, st.tier_offs, len(ids), self.H, cfg.batch_size, st.counts,
                                                first_batch=st.first_batch, stream=head)
            head_ctx.build_cache(st.counts, self.wl.home, None if self.prefetch else self.wl.remote_store, cfg.feat_dim,
                                 st.cache, stream=head)
            if self.planned:
                st.plan.set_num_batches(len(ids))
                head_ctx.plan_prefetch(st.cache, self.wl.home, st.first_batch, st.plan, stream=head)
            st.built.record(head)
        st.n_batches = len(ids)
        st.sizes = None
        st.pulls_queued = self.mirror

    def _call_sizes(self, n, gsz, first, last):
        """Batches per sampler call for the n batches of one epoch of a period.  Groups of gsz, except that with one pull
        per call the period opens with a single batch (its rows start crossing the link while the next calls sample)
        and closes with calls of 2, 1 and 1 batches (the gathers of a call's batches wait for its pull, so a short
        last pull leaves a short tail behind the link's last byte)."""
        if not self.group_pulls or gsz == 1:
            return [min(gsz, n - i) for i in range(0, n, gsz)]
        head = [1] if first and n > 1 else []
        tail = []
        if last:
            for size in (1, 1, 2):
                if sum(head) + sum(tail) + size < n:
                    tail.insert(0, size)
        body = n - sum(head) - sum(tail)
        return head + [min(gsz, body - i) for i in range(0, body, gsz)] + tail

    def precompute(self, epoch, n_batches=None, batch_ids=None):
        """Offline stage (asynchronous) for the first n_batches batches of `epoch`, or for the listed
        batch indices; slot i of the arena holds the i-th of them.  With period_epochs = E the same batches of the
        E epochs starting at `epoch` follow each other, epoch by epoch.  Uses every sampler lane."""
        ids = list(batch_ids) if batch_ids is not None else list(range(n_batches))
        assert len(ids) * self.period_epochs <= self.max_batches and all(0 <= b < self.batches_per_epoch for b in ids)
        lanes = [(self.lane_ctx[k], self.lane_bufs[k], self.lane_stream[k]) for k in range(self.n_lanes)]
        self._offline(self.state, epoch, ids, lanes)

    def read_sizes(self):
        """Every batch's input-node count on the host: waits for the copy queued right behind the sampling (not for
        the rest of the offline stage)."""
        st = self.state
        st.sizes_ready.synchronize()
        st.sizes = st.sizes_host[:st.n_batches, self.H + 1].tolist()
        return st.sizes

    def sampled_edges(self):
        """Total number of sampled edges over the precomputed batches (synchronises)."""
        return int(self.edge_counts[:self.n_batches].sum().item())

    # ---- online stage
    def gather(self, b):
        """Features of batch b's input nodes into self.out[:n]."""
        st = self.state
        n = st.sizes[b]
        main = torch.cuda.current_stream()
        q = self._gathered % self.queue_depth
        self._gathered += 1
        self.out = self.out_ring[q]
        if self.consumer:
            main.wait_event(self.consumed[q])           # the ring slot is free once its previous batch was consumed
        # the lookups of a whole group of batches are made by one launch (prepare); each batch then costs one copy
        # kernel on this stream (plus its miss rows on the miss stream)
        ticket = b % B.RG_GATHER_TICKETS
        if self._tickets.get(ticket) != (id(st), b):
            self._prepare(st, [b])
        # With a cache that can hold the whole remote partition no batch has miss rows once its pulls are done, so the
        # (empty) miss pass stays on this stream: the fork to the miss stream and the join back cost every gather more
        # than the pass itself.
        if self.decoupled:
            side, args = self.side, (n, st.cache, self.wl.local_store, self.wl.remote_store, self.cfg.feat_dim, self.out)
            half = self._fork_due.pop(ticket, None)
            if half is not None:
                side.wait_event(self.prep_done[half])   # the one fork of the group: the miss stream reads the lookups' lists
            side.wait_event(self.rows_done[q])          # the buffer's earlier batch: its HBM half (its miss half ran on this stream)
            if self.consumer:
                side.wait_event(self.consumed[q])
            self.ctx.gather_run_part(ticket, B.RG_GATHER_PART_MISS, *args, stream=side)
            self.miss_done[q].record(side)
            self.ctx.gather_run_part(ticket, B.RG_GATHER_PART_HBM, *args, stream=main)
            self.rows_done[q].record(main)
            main.wait_event(self.miss_done[q])          # the batch is whole on this stream
        else:
            self.ctx.gather_run(ticket, n, st.cache, self.wl.local_store, self.wl.remote_store, self.cfg.feat_dim, self.out,
                                hit_stream=main, miss_stream=main if self.no_misses else self.side)
        self._tickets.pop(ticket, None)
        if self.consumer:
            self.ready[q].record(main)
            cs = self.consumer_stream
            cs.wait_event(self.ready[q])
            blk_indptr, _, blk_nbr_local = st.blk[self.H - 1]
            self.ctx.mean_aggregate(blk_indptr[b], blk_nbr_local[b], self.bufs.frontier_ub[self.H - 1], self.out,
                                    self.cfg.feat_dim, self.agg, n_dst_dev=st.tier_offs[b, self.H:], stream=cs)
            self.consumed[q].record(cs)
        return n

    def _prepare(self, st, batches):
        """Classify the listed batches (consecutive, within one group of tickets) with one launch on the current stream."""
        first = batches[0] % B.RG_GATHER_TICKETS
        self.ctx.gather_prepare(first, [st.arena[b] for b in batches], [st.sizes[b] for b in batches], st.cache,
                                [st.stats[b] for b in batches])
        for b in batches:
            self._tickets[b % B.RG_GATHER_TICKETS] = (id(st), b)
        if self.decoupled:                              # the miss stream waits for it when it reaches the group's first batch
            half = (first * 2) // B.RG_GATHER_TICKETS
            self.prep_done[half].record(torch.cuda.current_stream())
            self._fork_due[first] = half

    def prefetch_rows(self, b, stream=None, st=None):
        """Pull the not-yet-resident cached rows batch b needs (asynchronous on `stream`).  The row count is
        read on the device, so the pulls of an epoch can be queued before the host knows its batch sizes."""
        st = st or self.state
        if self.planned:
            self.ctx.prefetch_planned(st.plan, b, st.cache, self.wl.remote_store, self.cfg.feat_dim, stream=stream)
            return
        self.ctx.prefetch_cache_rows(st.arena[b], self.slot, st.cache, self.wl.home, self.wl.remote_store,
                                     self.cfg.feat_dim, n_dev=st.tier_offs[b, self.H + 1:], stream=stream)

    def _queue_pulls(self, st):
        """All of an epoch's pulls on the prefetch stream, behind its TopHot, one event per batch."""
        if st.pulls_queued:
            return
        self.pf_stream.wait_event(st.built)
        for b in range(st.n_batches):
            self.prefetch_rows(b, stream=self.pf_stream, st=st)
            st.pf_events[b].record(self.pf_stream)
        st.pulls_queued = True

    def online(self, n_batches, on_batch=None):
        """Gathers in batch order; with prefetch on, batch b's gather waits only for the pulls of batches
        0..b, which run ahead on the prefetch stream.  on_batch(pipeline, b) is called after batch b's gather
        has been queued (the consumer of self.out[:n]; it must order itself after the current stream)."""
        st = self.state
        main = torch.cuda.current_stream()
        if self.prefetch and not st.pulls_queued:
            self.pf_stream.wait_stream(main)
        main.wait_event(st.built)                       # the offline stage may have run on other streams
        # Lookups are made for a group of batches at a time.  With decoupled misses the groups are half the tickets and
        # the lookups of the next group are queued before the current group's gathers (its tickets are those of the
        # group before, which is complete), so the miss stream finds the next group's lists ready when it gets there.
        G = B.RG_GATHER_TICKETS // 2 if self.decoupled else B.RG_GATHER_TICKETS
        group_of = lambda b0: list(range(b0, min(b0 + G, n_batches)))
        for b in range(n_batches):
            if b % G == 0:
                if not self.decoupled or b == 0:
                    self._prepare(st, group_of(b))
                if self.decoupled and b + G < n_batches:
                    self._prepare(st, group_of(b + G))
            if self.prefetch:
                if not st.pulls_queued:
                    self.prefetch_rows(b, stream=self.pf_stream)
                    st.pf_events[b].record(self.pf_stream)
                main.wait_event(st.pf_events[b])
            self.gather(b)
            if on_batch:
                on_batch(self, b)
        if self.prefetch:
            st.pulls_queued = True
        if self.consumer:
            main.wait_stream(self.consumer_stream)      # the epoch is served when its last batch has been consumed
        st.served.record(main)

    def run_epoch(self, epoch, n_batches, on_batch=None):
        """One period (period_epochs epochs of n_batches batches each) from a cold start: offline stage, size
        read-back, online stage."""
        self.precompute(epoch, n_batches)
        self.read_sizes()
        self.online(n_batches * self.period_epochs, on_batch)

    def run_epochs(self, first_epoch, n_periods, n_batches, on_epoch_done=None, on_batch=None, on_epoch_start=None):
        """Several periods back to back (a period is one epoch unless period_epochs says otherwise; the callbacks get
        the period's index).  With double buffering, period p+1 is precomputed on the build stream (one sampler lane)
        and its rows are pulled behind period p's while period p is being served."""
        E = self.period_epochs
        if not self.double_buffer or n_periods == 1:
            for k in range(n_periods):
                self.precompute(first_epoch + k * E, n_batches)
                self.read_sizes()
                if on_epoch_start:
                    on_epoch_start(self, k)
                self.online(n_batches * E, on_batch)
                if on_epoch_done:
                    on_epoch_done(self, k)
            return
        main = torch.cuda.current_stream()
        ids = list(range(n_batches))
        self.precompute(first_epoch, n_batches)                      # cold start: every lane
        build_lane = [(self.lane_ctx[1], self.lane_bufs[1], self.build_stream)]
        for k in range(n_periods):
            self.read_sizes()
            if self.prefetch:
                self._queue_pulls(self.state)
            nxt = self.states[1 - self.cur]
            if k + 1 < n_periods:
                # the other buffer set is free once the period that used it has been served
                self.build_stream.wait_event(nxt.served)
                self.build_stream.wait_stream(main)                  # and after anything already queued that reads the orders
                self._offline(nxt, first_epoch + (k + 1) * E, ids, build_lane)
            if on_epoch_start:
                on_epoch_start(self, k)
            self.online(n_batches * E, on_batch)
            if k + 1 < n_periods and self.prefetch:
                self._queue_pulls(nxt)                               # behind this period's pulls on the prefetch stream
            if on_epoch_done:
                on_epoch_done(self, k)
            self.cur = 1 - self.cur
        self.cur = 1 - self.cur                                      # leave the last served period current
