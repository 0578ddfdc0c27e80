"""CPU oracle of the A3GNN mini-batch path: TEST INFRASTRUCTURE ONLY.

Only tests, the smoke entry and the benchmark's cpu_baseline leg may import
this package; the GPU library never does.  The arithmetic lives in
a3_oracle.cpp; this module only marshals numpy arrays through ctypes.
"""
from .binding import (  # noqa: F401
    philox4x32_10, draw, fixlog2_q32, key, select, sample_blocks, gather_features, block_mean, count_accesses, rank_cache,
    cache_fifo_update, OracleBlocks,
)
