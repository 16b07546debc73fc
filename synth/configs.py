"""Named workload presets: the five synthetic configurations this build is measured on.

Shapes for "dense_social" and "sparse_copurchase" are the node / edge / feature
shapes of the two public graphs the paper evaluates on (its Table I); the graphs
themselves are synthetic power-law stand-ins, not the datasets.
"""
from dataclasses import dataclass
from typing import Optional, Tuple


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    num_nodes: int
    mean_degree: float          # target directed edges / nodes (realised is a few % lower)
    gamma: float                # power-law degree exponent of the Chung-Lu weights
    feat_dim: int
    fanouts: Tuple[int, ...]    # fanouts[h] applies to hop h counted outward from the seeds
    batch_size: int
    train_frac: float
    epochs: int
    partition: str              # "mod2" | "random4" | "mod4" | "groups4" (local = planted group 0)
    cache_frac: Optional[float]  # fraction of remote rows; None -> cache_bytes governs
    cache_bytes: Optional[int] = None
    offsets64: bool = False     # CSR row offsets as int64
    max_batches: Optional[int] = None  # only the first max_batches of each epoch are used
    num_classes: int = 2
    communities: int = 0        # > 0: planted groups in the graph (degree-corrected planted partition)
    p_in: float = 0.0           # probability that an edge's second endpoint is drawn inside the first one's group
    local_seeds: bool = False   # train ids are restricted to the local partition (one trainer per partition)

    def cache_capacity_rows(self, n_remote: int) -> int:
        if self.cache_frac is not None:
            return int(self.cache_frac * n_remote)          # floor
        return int(self.cache_bytes // (4 * self.feat_dim))

    def tier_upper_bounds(self):
        """Static upper bound on the cumulative frontier size after each hop."""
        out = [self.batch_size]
        for f in self.fanouts:
            out.append(min(self.num_nodes, out[-1] * (1 + f)))
        return out


CONFIGS = {
    "tiny": WorkloadConfig(
        name="tiny", num_nodes=10_000, mean_degree=20, gamma=2.1, feat_dim=64,
        fanouts=(10, 5), batch_size=256, train_frac=0.60, epochs=2,
        partition="mod2", cache_frac=0.10, max_batches=4),
    "small": WorkloadConfig(
        name="small", num_nodes=200_000, mean_degree=50, gamma=2.1, feat_dim=128,
        fanouts=(25, 10), batch_size=1024, train_frac=0.60, epochs=1,
        partition="random4", cache_frac=0.15),
    "dense_social": WorkloadConfig(
        name="dense_social", num_nodes=232_965, mean_degree=492, gamma=2.1, feat_dim=602,
        fanouts=(25, 10), batch_size=1024, train_frac=0.66, epochs=2,
        partition="mod4", cache_frac=0.20, num_classes=41),
    "sparse_copurchase": WorkloadConfig(
        name="sparse_copurchase", num_nodes=2_449_029, mean_degree=50.5, gamma=2.1, feat_dim=100,
        fanouts=(15, 10, 5), batch_size=1024, train_frac=0.08, epochs=2,
        partition="mod4", cache_frac=0.20, num_classes=47),
    "stress": WorkloadConfig(
        name="stress", num_nodes=10_000_000, mean_degree=50, gamma=2.0, feat_dim=256,
        fanouts=(15, 10, 5), batch_size=4096, train_frac=0.10, epochs=1,
        partition="mod4", cache_frac=None, cache_bytes=48_000_000_000, offsets64=True),
}


EXTRA_CONFIGS = {
    # Two more presets, outside the five measured configurations: the `small` shapes on a graph with four planted
    # groups, once partitioned at random and once along the groups (a stand-in for an edge-cut-minimising
    # partitioner), seeds taken from the local partition as a trainer does.  They show how much of the remote traffic
    # the partitioner removes before the cache sees it.
    "small_groups_random": WorkloadConfig(
        name="small_groups_random", num_nodes=200_000, mean_degree=50, gamma=2.1, feat_dim=128,
        fanouts=(25, 10), batch_size=1024, train_frac=0.60, epochs=1,
        partition="random4", cache_frac=0.15, communities=4, p_in=0.85, local_seeds=True),
    "small_groups_local": WorkloadConfig(
        name="small_groups_local", num_nodes=200_000, mean_degree=50, gamma=2.1, feat_dim=128,
        fanouts=(25, 10), batch_size=1024, train_frac=0.60, epochs=1,
        partition="groups4", cache_frac=0.15, communities=4, p_in=0.85, local_seeds=True),
}


def get_config(name: str) -> WorkloadConfig:
    if name in CONFIGS:
        return CONFIGS[name]
    if name in EXTRA_CONFIGS:
        return EXTRA_CONFIGS[name]
    raise KeyError(f"unknown workload {name!r}; choose from {sorted(CONFIGS) + sorted(EXTRA_CONFIGS)}")
