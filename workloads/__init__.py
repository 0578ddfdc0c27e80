"""Seeded synthetic inputs for the A3GNN mini-batch path.

Serves the CPU oracle's tests and the GPU library's tests / benchmark alike.
Nothing here is part of the method: no sampling keys, no selection, no
relabelling, no gather.  Only graphs, feature tables, cache splits and seed
batches, generated from integer hashes so that a given (config, seed) always
yields the same arrays on a given device type.
"""
from .graphs import powerlaw_degrees, chung_lu_csr, make_graph, Graph  # noqa: F401
from .features import make_features, degree_ranked_cache, padded_rows, CacheSplit, seed_batch  # noqa: F401
from .configs import CONFIGS, Workload, get_config  # noqa: F401
