"""Thin ctypes binding of librapidgnn.so: argument marshalling only.

Function names mirror the C ABI (include/rapidgnn.h).  Tensors are torch tensors that own
the device (or pinned host) memory; every step of the path runs inside the library's HIP
kernels.  There is no fallback: if the shared library is missing or cannot be loaded the
import of this module raises.
"""
import ctypes
import os

import torch  # noqa: F401  (loaded first so the HIP runtime already in the process is shared)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librapidgnn.so")

RG_OK, RG_ERR_INVALID_ARG, RG_ERR_CAPACITY, RG_ERR_OOM, RG_ERR_HIP, RG_ERR_STATE = range(6)
RG_MAX_FANOUT = 1024
RG_FANOUT_ALL = -1
RG_MAX_HOPS = 8
RG_MAX_GROUP = 16
RG_GATHER_TICKETS = 8
RG_ORDER_ASCENDING, RG_ORDER_FIRST_SEEN = 0, 1
RG_STATIC_GATHER_MAX_ROWS = 1 << 20
RG_GATHER_PART_HBM, RG_GATHER_PART_MISS = 1, 2
RG_K_GATHER_HBM, RG_K_GATHER_MISS, RG_K_SAMPLE, RG_K_HISTOGRAM, RG_K_CACHE_FILL, RG_K_AGGREGATE = range(6)

_STATUS_NAMES = {0: "RG_OK", 1: "RG_ERR_INVALID_ARG", 2: "RG_ERR_CAPACITY", 3: "RG_ERR_OOM",
                 4: "RG_ERR_HIP", 5: "RG_ERR_STATE"}

c_i64, c_i32, c_u64, c_u32 = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_uint32
c_p = ctypes.c_void_p


class RgError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{_STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


class rg_csr(ctypes.Structure):
    _fields_ = [("num_nodes", c_i64), ("num_edges", c_i64), ("row_ptr", c_p),
                ("row_ptr_bits", c_i32), ("col_idx", c_p)]


class rg_blocks(ctypes.Structure):
    _fields_ = [("nodes", c_p), ("nodes_cap", c_i64), ("tier_off", c_p),
                ("indptr", ctypes.POINTER(c_p)), ("indptr_cap", ctypes.POINTER(c_i64)),
                ("nbr", ctypes.POINTER(c_p)), ("nbr_local", ctypes.POINTER(c_p)),
                ("nbr_cap", ctypes.POINTER(c_i64)), ("num_edges", c_p)]


class rg_cache(ctypes.Structure):
    _fields_ = [("cache_ids", c_p), ("cache_rows", c_p), ("capacity_rows", c_i64),
                ("row_stride", c_i64), ("loc", c_p), ("num_cached", c_p), ("filled", c_p),
                ("mirror_rows", c_i64), ("home", c_p)]


class rg_prefetch_plan(ctypes.Structure):
    _fields_ = [("list", c_p), ("list_capacity", c_i64), ("offsets", c_p), ("num_batches", c_i32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                          "(python -m paper_2505_10806_amd.build); there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    L.rg_create.argtypes = [ctypes.c_int, ctypes.POINTER(c_p)]
    L.rg_destroy.argtypes = [c_p]
    L.rg_destroy.restype = None
    L.rg_last_error.argtypes = [c_p]
    L.rg_last_error.restype = ctypes.c_char_p
    L.rg_version.argtypes = []
    L.rg_version.restype = ctypes.c_char_p
    L.rg_reserve.argtypes = [c_p, c_i64, c_i64, c_i64, c_i32]
    L.rg_epoch_schedule.argtypes = [c_p, c_p, c_i64, c_u64, c_u32, c_p, c_p]
    L.rg_blocks_bounds.argtypes = [c_i64, c_i64, c_i64, c_p, c_i32, c_p, c_p]
    L.rg_sample_blocks.argtypes = [c_p, ctypes.POINTER(rg_csr), c_p, c_i32, c_p, c_i32, c_u64, c_u32,
                                   ctypes.POINTER(rg_blocks), c_p]
    L.rg_sample_blocks_group.argtypes = [c_p, ctypes.POINTER(rg_csr), c_i32, ctypes.POINTER(c_p), ctypes.POINTER(c_i32), c_p,
                                         c_i32, c_u64, c_u32, c_i32, ctypes.POINTER(rg_blocks), c_p]
    L.rg_access_histogram_sampled.argtypes = [c_p, c_i32, c_p, c_p, c_p, c_i64, c_p]
    L.rg_access_histogram.argtypes = [c_p, c_p, c_i64, c_p, c_p, c_i64, c_p]
    L.rg_access_histogram_epoch.argtypes = [c_p, c_p, c_i64, c_p, c_i32, c_i32, c_i32, c_p, c_p, c_i64, c_p]
    L.rg_plan_prefetch.argtypes = [c_p, ctypes.POINTER(rg_cache), c_p, c_p, c_i64, ctypes.POINTER(rg_prefetch_plan), c_p]
    L.rg_stream_create.argtypes = [c_p, c_i32, c_i32, ctypes.POINTER(c_p)]
    L.rg_stream_destroy.argtypes = [c_p, c_p]
    L.rg_plan_sampled.argtypes = [c_p, c_i32, ctypes.POINTER(rg_cache), c_p, ctypes.POINTER(rg_prefetch_plan), c_i32, c_i64, c_p]
    L.rg_prefetch_planned.argtypes = [c_p, ctypes.POINTER(rg_prefetch_plan), c_i32, ctypes.POINTER(rg_cache), c_p, c_i64, c_i32, c_p]
    L.rg_build_cache.argtypes = [c_p, c_p, c_p, c_i64, c_p, c_i64, c_i32, ctypes.POINTER(rg_cache), c_p]
    L.rg_cache_hit_curve.argtypes = [c_p, c_p, c_p, c_i64, c_p, c_i32, c_p, c_p, c_p]
    L.rg_prefetch_cache_rows.argtypes = [c_p, c_p, c_i64, c_p, ctypes.POINTER(rg_cache), c_p, c_p, c_i64, c_i32, c_p]
    L.rg_gather_prepare.argtypes = [c_p, c_i32, c_i32, ctypes.POINTER(c_p), ctypes.POINTER(c_i64), ctypes.POINTER(c_p),
                                    ctypes.POINTER(rg_cache), ctypes.POINTER(c_p), c_p]
    L.rg_gather_run.argtypes = [c_p, c_i32, c_i64, c_p, ctypes.POINTER(rg_cache), c_p, c_i64, c_p, c_i64, c_i32, c_p, c_i64,
                                c_p, c_p]
    L.rg_mean_aggregate.argtypes = [c_p, c_p, c_p, c_i64, c_p, c_p, c_i64, c_i32, c_p, c_i64, c_p]
    L.rg_gather_features.argtypes = [c_p, c_p, c_i64, c_p, ctypes.POINTER(rg_cache), c_p, c_i64, c_p, c_i64,
                                     c_i32, c_p, c_i64, c_p, c_p, c_p]
    L.rg_gather_features_static.argtypes = L.rg_gather_features.argtypes
    L.rg_gather_run_part.argtypes = [c_p, c_i32, c_i32, c_i64, c_p, ctypes.POINTER(rg_cache), c_p, c_i64, c_p, c_i64, c_i32, c_p, c_i64, c_p]
    L.rg_profile_enable.argtypes = [c_p, ctypes.c_int]
    L.rg_profile_reset.argtypes = [c_p]
    L.rg_profile_select.argtypes = [c_p, ctypes.c_uint32]
    L.rg_profile_read.argtypes = [c_p, ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(c_i64)]
    for name in ("rg_create", "rg_reserve", "rg_epoch_schedule", "rg_blocks_bounds", "rg_sample_blocks", "rg_sample_blocks_group",
                 "rg_access_histogram", "rg_access_histogram_epoch", "rg_access_histogram_sampled", "rg_build_cache", "rg_cache_hit_curve",
                 "rg_prefetch_cache_rows", "rg_plan_prefetch", "rg_plan_sampled", "rg_prefetch_planned", "rg_gather_features",
                 "rg_gather_features_static", "rg_gather_prepare", "rg_gather_run", "rg_mean_aggregate", "rg_profile_enable",
                 "rg_profile_reset", "rg_profile_read", "rg_profile_select", "rg_stream_create", "rg_stream_destroy", "rg_gather_run_part"):
        getattr(L, name).restype = ctypes.c_int
    return L


_lib = _load()

EXPORTED_SYMBOLS = ["rg_create", "rg_destroy", "rg_last_error", "rg_version", "rg_reserve", "rg_epoch_schedule",
                    "rg_blocks_bounds", "rg_sample_blocks", "rg_sample_blocks_group", "rg_access_histogram",
                    "rg_access_histogram_epoch", "rg_access_histogram_sampled",
                    "rg_build_cache", "rg_cache_hit_curve", "rg_prefetch_cache_rows", "rg_plan_prefetch",
                    "rg_plan_sampled", "rg_prefetch_planned", "rg_gather_features", "rg_gather_features_static",
                    "rg_stream_create", "rg_stream_destroy", "rg_gather_prepare", "rg_gather_run_part",
                    "rg_gather_run", "rg_mean_aggregate", "rg_profile_enable", "rg_profile_select", "rg_profile_reset", "rg_profile_read"]


def _ptr(t, dtype=None, device_type=None, name="tensor"):
    """Raw address of a contiguous tensor (None -> NULL)."""
    if t is None:
        return None
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if device_type is not None and t.device.type != device_type and not (device_type == "mapped"):
        raise ValueError(f"{name}: expected a {device_type} tensor, got {t.device}")
    if device_type == "mapped" and t.device.type != "cuda" and not t.is_pinned():
        raise ValueError(f"{name}: host tensor must be pinned to be read from the device")
    if not t.is_contiguous():
        raise ValueError(f"{name}: tensor must be contiguous")
    return t.data_ptr()


def _stream_handle(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


class Context:
    """Owns an rg_ctx.  Methods carry the C names without the rg_ prefix."""

    def __init__(self, device=0):
        h = c_p()
        st = _lib.rg_create(int(device), ctypes.byref(h))
        if st != RG_OK:
            raise RgError(st, _lib.rg_last_error(None).decode())
        self._h = h
        self.device = int(device)

    def close(self):
        if getattr(self, "_h", None):
            _lib.rg_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st):
        if st != RG_OK:
            raise RgError(st, _lib.rg_last_error(self._h).decode())

    # -- rg_reserve
    def reserve(self, num_nodes, max_frontier, max_rows, sample_group=1):
        self._check(_lib.rg_reserve(self._h, int(num_nodes), int(max_frontier), int(max_rows), int(sample_group)))

    # -- rg_epoch_schedule
    def epoch_schedule(self, train_ids, seed, epoch, order_out=None, stream=None):
        n = train_ids.numel()
        if order_out is None:
            order_out = torch.empty_like(train_ids)
        self._check(_lib.rg_epoch_schedule(self._h, _ptr(train_ids, torch.int32, "cuda", "train_ids"), n,
                                           int(seed), int(epoch), _ptr(order_out, torch.int32, "cuda", "order_out"),
                                           _stream_handle(stream)))
        return order_out

    # -- rg_sample_blocks
    def sample_blocks(self, csr, seeds, num_seeds, fanouts, seed, epoch, out, stream=None):
        """csr: CsrGraph; seeds: int32 cuda tensor; out: BlockBuffers."""
        fo = (c_i32 * len(fanouts))(*[int(f) for f in fanouts])
        self._check(_lib.rg_sample_blocks(self._h, ctypes.byref(csr.c_struct), _ptr(seeds, torch.int32, "cuda", "seeds"),
                                          int(num_seeds), fo, len(fanouts), int(seed), int(epoch),
                                          ctypes.byref(out.c_struct), _stream_handle(stream)))

    # -- rg_sample_blocks_group
    def sample_blocks_group(self, csr, seeds, fanouts, seed, epoch, outs, stream=None, node_order=RG_ORDER_ASCENDING):
        """seeds: list of int32 cuda tensors (one per batch); outs: list of BlockBuffers of the same length."""
        g = len(seeds)
        if g != len(outs) or not 1 <= g <= RG_MAX_GROUP:
            raise ValueError(f"sample_blocks_group: between 1 and {RG_MAX_GROUP} batches with one BlockBuffers each")
        ptrs = (c_p * g)(*[_ptr(t, torch.int32, "cuda", "seeds") for t in seeds])
        nums = (c_i32 * g)(*[t.numel() for t in seeds])
        structs = (rg_blocks * g)(*[o.c_struct for o in outs])
        fo = (c_i32 * len(fanouts))(*[int(f) for f in fanouts])
        status = _lib.rg_sample_blocks_group(self._h, ctypes.byref(csr.c_struct), g, ptrs, nums, fo, len(fanouts),
                                             int(seed), int(epoch), int(node_order), structs, _stream_handle(stream))
        if status == RG_ERR_CAPACITY:      # the required sizes came back in the structs (the per-hop arrays are shared)
            for o, st in zip(outs, structs):
                o.c_struct.nodes_cap = st.nodes_cap
        self._check(status)

    # -- rg_access_histogram
    def access_histogram(self, nodes, n, counts, n_dev=None, stream=None):
        self._check(_lib.rg_access_histogram(self._h, _ptr(nodes, torch.int32, "cuda", "nodes"), int(n),
                                             _ptr(n_dev, torch.int32, "cuda", "n_dev"),
                                             _ptr(counts, torch.int32, "cuda", "counts"), counts.numel(),
                                             _stream_handle(stream)))

    # -- rg_access_histogram_sampled
    def access_histogram_sampled(self, group, counts, batch_index=None, first_batch=None, stream=None):
        idx = None if batch_index is None else (c_i32 * group)(*[int(b) for b in batch_index])
        self._check(_lib.rg_access_histogram_sampled(self._h, int(group), idx, _ptr(counts, torch.int32, "cuda", "counts"),
                                                     _ptr(first_batch, torch.int32, "cuda", "first_batch"), counts.numel(),
                                                     _stream_handle(stream)))

    # -- rg_access_histogram_epoch
    def access_histogram_epoch(self, arena, tier_offs, num_batches, num_hops, max_seeds, counts, first_batch=None,
                               stream=None):
        """arena: int32 [>= num_batches, batch_stride]; tier_offs: int32 [>= num_batches, num_hops + 2];
        first_batch: optional int32 [num_nodes] preset to -1 (= 0xFFFFFFFF)."""
        if tier_offs.dim() != 2 or tier_offs.shape[1] != num_hops + 2 or arena.dim() != 2:
            raise ValueError("access_histogram_epoch: arena must be 2-D and tier_offs [batches, num_hops + 2]")
        if num_batches > arena.shape[0] or num_batches > tier_offs.shape[0]:
            raise ValueError("access_histogram_epoch: num_batches exceeds the buffers")
        self._check(_lib.rg_access_histogram_epoch(
            self._h, _ptr(arena, torch.int32, "cuda", "arena"), arena.stride(0),
            _ptr(tier_offs, torch.int32, "cuda", "tier_offs"), int(num_batches), int(num_hops), int(max_seeds),
            _ptr(counts, torch.int32, "cuda", "counts"), _ptr(first_batch, torch.int32, "cuda", "first_batch"),
            counts.numel(), _stream_handle(stream)))

    # -- rg_plan_prefetch / rg_prefetch_planned
    def plan_prefetch(self, cache, home, first_batch, plan, stream=None):
        self._check(_lib.rg_plan_prefetch(self._h, ctypes.byref(cache.c_struct), _ptr(home, torch.int32, "cuda", "home"),
                                          _ptr(first_batch, torch.int32, "cuda", "first_batch"), home.numel(),
                                          ctypes.byref(plan.c_struct), _stream_handle(stream)))

    def stream_on_cus(self, first_cu, num_cus):
        """A torch stream whose kernels run only on compute units [first_cu, first_cu + num_cus).  It belongs to this
        context and goes with it (or with rg_stream_destroy): by then nothing may refer to it any more, neither events
        recorded on it nor pinned tensors copied on it (torch records an event on their streams when they are freed).
        Pipelines take theirs from shared_stream_on_cus, which keeps them for the life of the process."""
        h = c_p()
        self._check(_lib.rg_stream_create(self._h, int(first_cu), int(num_cus), ctypes.byref(h)))
        return torch.cuda.ExternalStream(h.value, device=torch.device("cuda", self.device))

    @property
    def num_cus(self):
        return torch.cuda.get_device_properties(self.device).multi_processor_count

    def plan_sampled(self, group, cache, claimed, plan, segment, stream=None):
        self._check(_lib.rg_plan_sampled(self._h, int(group), ctypes.byref(cache.c_struct),
                                         _ptr(claimed, torch.int32, "cuda", "claimed"), ctypes.byref(plan.c_struct), int(segment),
                                         cache.loc.numel(), _stream_handle(stream)))

    def prefetch_planned(self, plan, batch, cache, remote_store, dim, stream=None):
        self._check(_lib.rg_prefetch_planned(self._h, ctypes.byref(plan.c_struct), int(batch), ctypes.byref(cache.c_struct),
                                             _ptr(remote_store, torch.float32, "mapped", "remote_store"),
                                             remote_store.stride(0), int(dim), _stream_handle(stream)))

    # -- rg_build_cache
    def build_cache(self, counts, home, remote_store, dim, cache, stream=None):
        """remote_store=None selects only (rows are pulled later by prefetch_cache_rows)."""
        rs = 0 if remote_store is None else (remote_store.stride(0) if remote_store.dim() == 2 else dim)
        self._check(_lib.rg_build_cache(self._h, _ptr(counts, torch.int32, "cuda", "counts"),
                                        _ptr(home, torch.int32, "cuda", "home"), home.numel(),
                                        _ptr(remote_store, torch.float32, "mapped", "remote_store"), rs, int(dim),
                                        ctypes.byref(cache.c_struct), _stream_handle(stream)))

    # -- rg_cache_hit_curve
    def cache_hit_curve(self, counts, home, capacities, stream=None):
        """Returns (hits int64 cuda tensor [len(capacities)], remote_total int64 cuda tensor [1])."""
        caps = (c_i64 * len(capacities))(*[int(c) for c in capacities])
        hits = torch.zeros(max(len(capacities), 1), dtype=torch.int64, device=counts.device)
        total = torch.zeros(1, dtype=torch.int64, device=counts.device)
        self._check(_lib.rg_cache_hit_curve(self._h, _ptr(counts, torch.int32, "cuda", "counts"),
                                            _ptr(home, torch.int32, "cuda", "home"), home.numel(), caps, len(capacities),
                                            hits.data_ptr(), total.data_ptr(), _stream_handle(stream)))
        return hits[:len(capacities)], total

    # -- rg_prefetch_cache_rows
    def prefetch_cache_rows(self, input_nodes, n, cache, home, remote_store, dim, n_dev=None, stream=None):
        self._check(_lib.rg_prefetch_cache_rows(
            self._h, _ptr(input_nodes, torch.int32, "cuda", "input_nodes"), int(n),
            _ptr(n_dev, torch.int32, "cuda", "n_dev"), ctypes.byref(cache.c_struct),
            _ptr(home, torch.int32, "cuda", "home"),
            _ptr(remote_store, torch.float32, "mapped", "remote_store"), remote_store.stride(0), int(dim),
            _stream_handle(stream)))

    # -- rg_gather_features
    def gather_features(self, input_nodes, n, cache, local_store, remote_store, dim, out, stats,
                        n_dev=None, hit_stream=None, miss_stream=None):
        self._check(_lib.rg_gather_features(
            self._h, _ptr(input_nodes, torch.int32, "cuda", "input_nodes"), int(n),
            _ptr(n_dev, torch.int32, "cuda", "n_dev"), ctypes.byref(cache.c_struct),
            _ptr(local_store, torch.float32, "cuda", "local_store"), local_store.stride(0),
            _ptr(remote_store, torch.float32, "mapped", "remote_store"), remote_store.stride(0),
            int(dim), _ptr(out, torch.float32, "cuda", "out"), out.stride(0),
            _ptr(stats, torch.int64, "cuda", "stats"), _stream_handle(hit_stream),
            None if miss_stream is None else _stream_handle(miss_stream)))

    # -- rg_gather_features_static
    def gather_features_static(self, input_nodes, n, cache, local_store, remote_store, dim, out, stats,
                               n_dev=None, hit_stream=None, miss_stream=None):
        self._check(_lib.rg_gather_features_static(
            self._h, _ptr(input_nodes, torch.int32, "cuda", "input_nodes"), int(n),
            _ptr(n_dev, torch.int32, "cuda", "n_dev"), ctypes.byref(cache.c_struct),
            _ptr(local_store, torch.float32, "cuda", "local_store"), local_store.stride(0),
            _ptr(remote_store, torch.float32, "mapped", "remote_store"), remote_store.stride(0),
            int(dim), _ptr(out, torch.float32, "cuda", "out"), out.stride(0),
            _ptr(stats, torch.int64, "cuda", "stats"), _stream_handle(hit_stream),
            None if miss_stream is None else _stream_handle(miss_stream)))

    # -- rg_gather_prepare / rg_gather_run
    def gather_prepare(self, first_ticket, input_nodes, n, cache, stats, n_dev=None, stream=None):
        """input_nodes, stats (and n_dev): lists with one tensor per batch; n: list of row counts."""
        g = len(input_nodes)
        nodes = (c_p * g)(*[_ptr(t, torch.int32, "cuda", "input_nodes") for t in input_nodes])
        rows = (c_i64 * g)(*[int(x) for x in n])
        sts = (c_p * g)(*[_ptr(t, torch.int64, "cuda", "stats") for t in stats])
        nd = None if n_dev is None else (c_p * g)(*[_ptr(t, torch.int32, "cuda", "n_dev") for t in n_dev])
        self._check(_lib.rg_gather_prepare(self._h, int(first_ticket), g, nodes, rows, nd, ctypes.byref(cache.c_struct), sts,
                                           _stream_handle(stream)))

    def gather_run(self, ticket, n, cache, local_store, remote_store, dim, out, n_dev=None, hit_stream=None,
                   miss_stream=None):
        self._check(_lib.rg_gather_run(
            self._h, int(ticket), int(n), _ptr(n_dev, torch.int32, "cuda", "n_dev"), ctypes.byref(cache.c_struct),
            _ptr(local_store, torch.float32, "cuda", "local_store"), local_store.stride(0),
            _ptr(remote_store, torch.float32, "mapped", "remote_store"), remote_store.stride(0),
            int(dim), _ptr(out, torch.float32, "cuda", "out"), out.stride(0), _stream_handle(hit_stream),
            None if miss_stream is None else _stream_handle(miss_stream)))

    def gather_run_part(self, ticket, part, n, cache, local_store, remote_store, dim, out, n_dev=None, stream=None):
        self._check(_lib.rg_gather_run_part(
            self._h, int(ticket), int(part), int(n), _ptr(n_dev, torch.int32, "cuda", "n_dev"), ctypes.byref(cache.c_struct),
            _ptr(local_store, torch.float32, "cuda", "local_store"), local_store.stride(0),
            _ptr(remote_store, torch.float32, "mapped", "remote_store"), remote_store.stride(0),
            int(dim), _ptr(out, torch.float32, "cuda", "out"), out.stride(0), _stream_handle(stream)))

    # -- rg_mean_aggregate
    def mean_aggregate(self, indptr, nbr_local, n_dst, feat, dim, agg, n_dst_dev=None, stream=None):
        self._check(_lib.rg_mean_aggregate(
            self._h, _ptr(indptr, torch.int32, "cuda", "indptr"), _ptr(nbr_local, torch.int32, "cuda", "nbr_local"),
            int(n_dst), _ptr(n_dst_dev, torch.int32, "cuda", "n_dst_dev"),
            _ptr(feat, torch.float32, "cuda", "feat"), feat.stride(0), int(dim),
            _ptr(agg, torch.float32, "cuda", "agg"), agg.stride(0), _stream_handle(stream)))

    # -- rg_profile_*
    def profile_enable(self, on=True):
        self._check(_lib.rg_profile_enable(self._h, 1 if on else 0))

    def profile_select(self, kernel_ids=None):
        """Bracket only the listed kernel ids while profiling is on (None = all)."""
        mask = 0xFFFFFFFF if kernel_ids is None else sum(1 << int(k) for k in set(kernel_ids))
        self._check(_lib.rg_profile_select(self._h, mask))

    def profile_reset(self):
        self._check(_lib.rg_profile_reset(self._h))

    def profile_read(self, kernel_id):
        ms = ctypes.c_double()
        cnt = c_i64()
        self._check(_lib.rg_profile_read(self._h, int(kernel_id), ctypes.byref(ms), ctypes.byref(cnt)))
        return ms.value, cnt.value


def blocks_bounds(num_nodes, num_edges, num_seeds, fanouts):
    """rg_blocks_bounds: (frontier_ub[H+1], edges_ub[H]) as Python lists."""
    H = len(fanouts)
    fo = (c_i32 * H)(*[int(f) for f in fanouts])
    fub = (c_i64 * (H + 1))()
    eub = (c_i64 * H)()
    st = _lib.rg_blocks_bounds(int(num_nodes), int(num_edges), int(num_seeds), fo, H, fub, eub)
    if st != RG_OK:
        raise RgError(st, "rg_blocks_bounds: invalid argument")
    return list(fub), list(eub)


def version():
    return _lib.rg_version().decode()


class CsrGraph:
    """rg_csr over two cuda tensors (kept alive by this object)."""

    def __init__(self, row_ptr, col_idx):
        if row_ptr.dtype not in (torch.int32, torch.int64):
            raise TypeError("row_ptr must be int32 or int64")
        self.row_ptr, self.col_idx = row_ptr, col_idx
        self.num_nodes = row_ptr.numel() - 1
        self.num_edges = col_idx.numel()
        self.c_struct = rg_csr(self.num_nodes, self.num_edges, _ptr(row_ptr, None, "cuda", "row_ptr"),
                               32 if row_ptr.dtype == torch.int32 else 64, _ptr(col_idx, torch.int32, "cuda", "col_idx"))


class BlockBuffers:
    """Caller-owned output buffers of rg_sample_blocks, sized by rg_blocks_bounds."""

    def __init__(self, num_nodes, num_edges, max_seeds, fanouts, device, with_local=True, nodes=None):
        self.fanouts = tuple(int(f) for f in fanouts)
        H = len(self.fanouts)
        self.frontier_ub, self.edges_ub = blocks_bounds(num_nodes, num_edges, max_seeds, self.fanouts)
        i32 = dict(dtype=torch.int32, device=device)
        self.nodes = nodes if nodes is not None else torch.empty(max(self.frontier_ub[H], 1), **i32)
        self.tier_off = torch.zeros(H + 2, **i32)
        self.num_edges = torch.zeros(H, **i32)
        self.indptr = [torch.empty(self.frontier_ub[h] + 1, **i32) for h in range(H)]
        self.nbr = [torch.empty(max(self.edges_ub[h], 1), **i32) for h in range(H)]
        self.nbr_local = [torch.empty(max(self.edges_ub[h], 1), **i32) for h in range(H)] if with_local else None
        self._build_struct()

    def _build_struct(self):
        H = len(self.fanouts)
        self._indptr_arr = (c_p * H)(*[t.data_ptr() for t in self.indptr])
        self._nbr_arr = (c_p * H)(*[t.data_ptr() for t in self.nbr])
        self._loc_arr = (c_p * H)(*[t.data_ptr() for t in self.nbr_local]) if self.nbr_local else None
        self._indptr_cap = (c_i64 * H)(*[t.numel() for t in self.indptr])
        self._nbr_cap = (c_i64 * H)(*[t.numel() for t in self.nbr])
        self.c_struct = rg_blocks(
            self.nodes.data_ptr(), self.nodes.numel(), self.tier_off.data_ptr(),
            ctypes.cast(self._indptr_arr, ctypes.POINTER(c_p)), ctypes.cast(self._indptr_cap, ctypes.POINTER(c_i64)),
            ctypes.cast(self._nbr_arr, ctypes.POINTER(c_p)),
            ctypes.cast(self._loc_arr, ctypes.POINTER(c_p)) if self._loc_arr is not None else None,
            ctypes.cast(self._nbr_cap, ctypes.POINTER(c_i64)), self.num_edges.data_ptr())

    def set_hop(self, h, indptr=None, nbr=None, nbr_local=None):
        """Point hop h's outputs at other buffers (e.g. to keep a batch's outermost block for its consumer)."""
        for name, t, arr, cap in (("indptr", indptr, self._indptr_arr, self._indptr_cap),
                                  ("nbr", nbr, self._nbr_arr, self._nbr_cap),
                                  ("nbr_local", nbr_local, self._loc_arr, self._nbr_cap)):
            if t is None:
                continue
            if t.dtype != torch.int32 or not t.is_contiguous() or arr is None:
                raise TypeError(f"set_hop: {name} must be a contiguous int32 tensor (and relabelling enabled for nbr_local)")
            need = self.frontier_ub[h] + 1 if name == "indptr" else self.edges_ub[h]
            if t.numel() < need:
                raise ValueError(f"set_hop: {name} holds {t.numel()} entries, {need} required")
            getattr(self, name)[h] = t
            arr[h] = t.data_ptr()
            if name != "nbr_local":
                cap[h] = t.numel()
        if nbr is not None and nbr_local is not None and nbr.numel() != nbr_local.numel():
            raise ValueError("set_hop: nbr and nbr_local must have the same capacity")

    def set_outputs(self, nodes, tier_off, num_edges=None):
        """Point the input-node list, tier offsets and per-hop edge counts at other buffers (e.g. a batch's slot
        of an epoch arena)."""
        if num_edges is not None:
            if num_edges.dtype != torch.int32 or num_edges.numel() < len(self.fanouts):
                raise TypeError("set_outputs: num_edges must be int32 with num_hops entries")
            self.num_edges = num_edges
            self.c_struct.num_edges = num_edges.data_ptr()
        if nodes.dtype != torch.int32 or tier_off.dtype != torch.int32 or tier_off.numel() < len(self.fanouts) + 2:
            raise TypeError("set_outputs: int32 tensors required, tier_off of num_hops + 2 entries")
        self.nodes, self.tier_off = nodes, tier_off
        self.c_struct.nodes = nodes.data_ptr()
        self.c_struct.nodes_cap = nodes.numel()
        self.c_struct.tier_off = tier_off.data_ptr()


# Streams bound to a share of the compute units, one per (device, range, role), kept for the life of the process: torch
# objects of any pipeline may refer to them (events, pinned buffers), so they are never destroyed while pipelines live.
_shared_streams = {}
_stream_owner = {}


def shared_stream_on_cus(device, first_cu, num_cus, role):
    """The process-wide stream of `role` (any hashable) on compute units [first_cu, first_cu + num_cus) of `device`."""
    device = int(device)
    key = (device, int(first_cu), int(num_cus), role)
    if key not in _shared_streams:
        if device not in _stream_owner:
            _stream_owner[device] = Context(device)
        _shared_streams[key] = _stream_owner[device].stream_on_cus(first_cu, num_cus)
    return _shared_streams[key]


def close_shared_streams():
    """Gives the shared streams back.  Only for a program's last lines, once every pipeline and every torch object that
    worked on them is gone (a profiler that wraps the runtime wants the streams destroyed before the process exits)."""
    import gc
    gc.collect()
    for device, owner in list(_stream_owner.items()):
        try:
            torch.cuda.synchronize(device)
        except Exception:
            pass
        owner.close()
    _shared_streams.clear()
    _stream_owner.clear()


class FeatureCache:
    """rg_cache over caller-owned cuda tensors."""

    def __init__(self, num_nodes, capacity_rows, row_stride, device, mirror_rows=0, home=None):
        """mirror_rows > 0 (with the home words): the cache holds the whole remote partition and is laid out as its
        mirror (row of a cached node = its remote-store row)."""
        self.capacity_rows = int(capacity_rows)
        if mirror_rows and (home is None or mirror_rows > self.capacity_rows):
            raise ValueError("a mirrored cache needs the home words and capacity_rows >= mirror_rows")
        self.mirror_rows, self.home = int(mirror_rows), home
        self.cache_ids = torch.empty(max(self.capacity_rows, 1), dtype=torch.int32, device=device)
        self.cache_rows = torch.empty(max(self.capacity_rows, 1), int(row_stride), dtype=torch.float32, device=device)
        self.loc = torch.empty(max(num_nodes, 1), dtype=torch.int32, device=device)
        self.num_cached = torch.zeros(1, dtype=torch.int64, device=device)
        self.filled = torch.zeros(max((min(self.capacity_rows, num_nodes) + 31) // 32, 1), dtype=torch.int32, device=device)
        self.c_struct = rg_cache(self.cache_ids.data_ptr(), self.cache_rows.data_ptr(), self.capacity_rows,
                                 int(row_stride), self.loc.data_ptr(), self.num_cached.data_ptr(), self.filled.data_ptr(),
                                 self.mirror_rows, _ptr(home, torch.int32, "cuda", "home") if self.mirror_rows else None)

    @classmethod
    def sharing_rows(cls, other, num_nodes, device):
        """A second mirrored cache (own ids, location table and count) over the rows and resident bits of `other`."""
        self = cls.__new__(cls)
        self.capacity_rows, self.mirror_rows, self.home = other.capacity_rows, other.mirror_rows, other.home
        if not self.mirror_rows:
            raise ValueError("only mirrored caches can share their rows")
        self.cache_ids = torch.empty_like(other.cache_ids)
        self.cache_rows, self.filled = other.cache_rows, other.filled
        self.loc = torch.empty(max(num_nodes, 1), dtype=torch.int32, device=device)
        self.num_cached = torch.zeros(1, dtype=torch.int64, device=device)
        self.c_struct = rg_cache(self.cache_ids.data_ptr(), self.cache_rows.data_ptr(), self.capacity_rows,
                                 other.c_struct.row_stride, self.loc.data_ptr(), self.num_cached.data_ptr(), self.filled.data_ptr(),
                                 self.mirror_rows, other.c_struct.home)
        return self

    def rows_of(self, node_ids):
        """Rows of cache_rows that hold the listed cached nodes (int64 cuda tensor), for either layout."""
        ids = node_ids.long()
        words = (self.home if self.mirror_rows else self.loc)[ids].long() & 0x3FFFFFFF
        return words


class PrefetchPlan:
    """rg_prefetch_plan over caller-owned cuda tensors."""

    def __init__(self, list_capacity, max_batches, device):
        self.list = torch.empty(2 * max(int(list_capacity), 1), dtype=torch.int32, device=device)
        self.offsets = torch.zeros(int(max_batches) + 2, dtype=torch.int32, device=device)
        self.max_batches = int(max_batches)
        self.c_struct = rg_prefetch_plan(self.list.data_ptr(), int(list_capacity), self.offsets.data_ptr(), int(max_batches))

    def set_num_batches(self, n):
        if not 0 <= n <= self.max_batches:
            raise ValueError("PrefetchPlan: num_batches exceeds the offsets buffer")
        self.c_struct.num_batches = int(n)
