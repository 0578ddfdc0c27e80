"""MI355X-native mini-batch path of A3GNN: locality-aware neighbour sampling, reindex into
per-hop block CSRs, and feature gather from an HBM cache plus a pinned-host remainder.

All computation happens in the HIP library behind the C ABI of include/a3gnn.h; this package
only marshals torch tensors (device memory, streams) into that ABI.
"""
from .binding import (  # noqa: F401
    A3Error, Context, Pipeline, Blocks, HostBlocks, lib, library_path,
    A3_PIPE_SEQUENTIAL, A3_PIPE_MODE1, A3_PIPE_MODE2, A3_PIPE_MAX_WORKERS, A3_F32, A3_F16,
    A3_OK, A3_ERR_INVALID_ARG, A3_ERR_CAPACITY, A3_ERR_HIP, A3_ERR_INPUT,
    A3_VALIDATE, A3_NO_EIDS, A3_HOST_ONLY, A3_FORCE_RADIX, A3_PROFILE, A3_TEST_MAP_RANGE, A3_TEST_FEW_DRAWS, A3_TEST_SMALL_GRID, A3_PROFILE_RETRIEVE, A3_STATIC_MAP, A3_PROFILE_DEPTH, A3_MAX_HOPS, A3_MAX_FANOUT,
    A3_FIFO_STATIC_MAX_IDS,
)
from .cpu_sampler import (  # noqa: F401
    CpuSampler, check_vector_forms, set_vector_form, set_first_bar_percent,
)
