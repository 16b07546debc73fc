"""Features, train split, partition and the packed feature stores of a workload.

Interface format shared with the library header and the oracle (an input/output
encoding, not arithmetic): a location word is ``(tag << 30) | row`` stored in an int32
array and read as uint32, tag 0 = local store (HBM), 1 = cache (HBM), 2 = remote store
(pinned host memory); ``row`` indexes rows of the named store.
"""
from dataclasses import dataclass
from typing import Optional

import torch

from .configs import WorkloadConfig, get_config
from .graph import chung_lu_csr

TAG_LOCAL, TAG_CACHE, TAG_REMOTE = 0, 1, 2
TAG_SHIFT = 30
ROW_MASK = (1 << TAG_SHIFT) - 1


def row_stride(dim: int) -> int:
    """Row stride in floats: rows padded to a multiple of 16 bytes."""
    return (dim + 3) // 4 * 4


def make_features(num_nodes, dim, seed, device="cpu"):
    gen = torch.Generator(device=torch.device(device))
    gen.manual_seed(int(seed) + 0x5EED0001)
    return torch.randn(num_nodes, dim, dtype=torch.float32, generator=gen, device=device)


def make_train_ids(num_nodes, frac, seed, device="cpu"):
    """First floor(frac*N) ids of a seeded permutation, as int32."""
    gen = torch.Generator(device=torch.device(device))
    gen.manual_seed(int(seed) + 0x5EED0002)
    perm = torch.randperm(num_nodes, generator=gen, device=device)
    return perm[: int(frac * num_nodes)].to(torch.int32).contiguous()


def make_partition(num_nodes, scheme, seed, device="cpu", groups=None):
    """Boolean mask of the nodes whose features are local (resident in HBM)."""
    ids = torch.arange(num_nodes, device=device)
    if scheme == "groups4":
        if groups is None:
            raise ValueError("partition 'groups4' needs the graph's planted group labels")
        return groups.to(device) == 0
    if scheme == "mod2":
        return ids % 2 == 0
    if scheme == "mod4":
        return ids % 4 == 0
    if scheme == "random4":
        gen = torch.Generator(device=torch.device(device))
        gen.manual_seed(int(seed) + 0x5EED0003)
        return torch.randint(0, 4, (num_nodes,), generator=gen, device=device) == 0
    raise ValueError(f"unknown partition scheme {scheme!r}")


def make_home(is_local):
    """home[v] = location word of v before any caching: rows packed in ascending id per store."""
    is_local = is_local.to(torch.bool)
    local_row = torch.cumsum(is_local, 0) - 1
    remote_row = torch.cumsum(~is_local, 0) - 1
    word = torch.where(is_local, local_row + (TAG_LOCAL << TAG_SHIFT), remote_row + (TAG_REMOTE << TAG_SHIFT))
    # store the uint32 bit pattern in an int32 tensor
    word = torch.where(word >= 2 ** 31, word - 2 ** 32, word)
    return word.to(torch.int32).contiguous()


def _pack(features, mask, stride, device, pinned):
    rows = features[mask.to(features.device)]
    n, d = rows.shape
    if pinned:
        out = torch.zeros(max(n, 1), stride, dtype=torch.float32, pin_memory=True)
    else:
        out = torch.zeros(max(n, 1), stride, dtype=torch.float32, device=device)
    out[:n, :d].copy_(rows)
    return out


@dataclass
class Workload:
    cfg: WorkloadConfig
    seed: int
    row_ptr: torch.Tensor            # int32 or int64 [N+1]
    col_idx: torch.Tensor            # int32 [nnz]
    features: Optional[torch.Tensor]  # fp32 [N, D], the unpartitioned matrix (may be dropped)
    train_ids: torch.Tensor          # int32 [n_train]
    is_local: torch.Tensor           # bool [N]
    home: torch.Tensor               # int32 [N] location words
    local_store: torch.Tensor        # fp32 [n_local, stride] on `device`
    remote_store: torch.Tensor       # fp32 [n_remote, stride] in (pinned) host memory
    stride: int
    n_local: int
    n_remote: int
    capacity_rows: int

    @property
    def num_nodes(self):
        return self.cfg.num_nodes

    @property
    def nnz(self):
        return int(self.col_idx.numel())

    def batches_per_epoch(self):
        n = int(self.train_ids.numel())
        full = -(-n // self.cfg.batch_size)          # the partial last batch is kept
        return full if self.cfg.max_batches is None else min(full, self.cfg.max_batches)


def build_workload(name_or_cfg, seed=2025, device="cpu", keep_features=True, pin_remote=None) -> Workload:
    """Generate every input of one named workload from a single master seed."""
    cfg = name_or_cfg if isinstance(name_or_cfg, WorkloadConfig) else get_config(name_or_cfg)
    device = torch.device(device)
    if pin_remote is None:
        pin_remote = device.type == "cuda"
    row_ptr, col_idx, groups = chung_lu_csr(cfg.num_nodes, cfg.mean_degree, cfg.gamma, seed, device, cfg.offsets64,
                                            communities=cfg.communities, p_in=cfg.p_in, return_communities=True)
    feats = make_features(cfg.num_nodes, cfg.feat_dim, seed, device)
    train_ids = make_train_ids(cfg.num_nodes, cfg.train_frac, seed, device)
    is_local = make_partition(cfg.num_nodes, cfg.partition, seed, device, groups)
    if cfg.local_seeds:          # a trainer draws its seeds from its own partition
        train_ids = train_ids[is_local[train_ids.long()]].contiguous()
    home = make_home(is_local)
    stride = row_stride(cfg.feat_dim)
    local_store = _pack(feats, is_local, stride, device, pinned=False)
    remote_store = _pack(feats, ~is_local, stride, "cpu", pinned=pin_remote)
    n_local = int(is_local.sum())
    n_remote = cfg.num_nodes - n_local
    return Workload(cfg=cfg, seed=seed, row_ptr=row_ptr, col_idx=col_idx,
                    features=feats if keep_features else None, train_ids=train_ids,
                    is_local=is_local, home=home, local_store=local_store,
                    remote_store=remote_store, stride=stride, n_local=n_local,
                    n_remote=n_remote, capacity_rows=cfg.cache_capacity_rows(n_remote))
