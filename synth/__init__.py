"""Seeded synthetic inputs shared by the CPU oracle tests, the GPU tests and bench.py.

This package only *produces inputs*: graphs, features, splits, partitions and the
packed feature stores.  It contains none of the method's arithmetic (no Philox, no
sampling rule, no histogram / top-K / gather logic) and imports neither the oracle
nor the HIP binding.  Random numbers come from torch's own generators.
"""
from .configs import CONFIGS, EXTRA_CONFIGS, WorkloadConfig, get_config  # noqa: F401
from .graph import chung_lu_csr  # noqa: F401
from .stores import (  # noqa: F401
    TAG_LOCAL, TAG_CACHE, TAG_REMOTE, TAG_SHIFT, ROW_MASK,
    Workload, build_workload, make_features, make_partition, make_train_ids,
)
