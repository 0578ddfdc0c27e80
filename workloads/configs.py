"""The five benchmark workloads (shapes only; synthetic stand-ins for the paper's datasets)
plus scaled-down variants that a CPU finishes in seconds."""
from dataclasses import dataclass, field
from typing import List

import torch


@dataclass
class Workload:
    name: str
    num_nodes: int
    mean_degree: float
    d_min: int
    d_max: int
    symmetric: bool
    idx_dtype: torch.dtype
    feat_dim: int
    feat_dtype: torch.dtype
    cache_frac: float
    batch: int
    fanouts: List[int]
    a: float = 2.1
    graph_seed: int = 0
    bias_rates: List[float] = field(default_factory=lambda: [1.0])

    @property
    def row_bytes(self) -> int:
        return self.feat_dim * torch.empty(0, dtype=self.feat_dtype).element_size()


CONFIGS = {
    # config 1: tiny graph, everything cached, 8 mini-batches rng_seed = 0..7
    "tiny": Workload("tiny", 10_000, 10.0, 1, 9_999, True, torch.int32, 64, torch.float32, 1.0,
                     256, [10, 5]),
    # config 2: dense social-style graph (Reddit-like shape), 602-dim fp32 rows, all in HBM
    "social": Workload("social", 232_965, 490.0, 1, 20_000, True, torch.int32, 602, torch.float32,
                       1.0, 1024, [25, 10]),
    # config 3: co-purchase-style graph (Products-like shape), top 20 % by degree cached
    "copurchase": Workload("copurchase", 2_450_000, 50.6, 1, 20_000, True, torch.int32, 100,
                           torch.float32, 0.2, 4096, [15, 10, 5], bias_rates=[1.0, 4.0]),
    # config 5: citation-scale graph, int64 indices, fp16 rows, all in HBM
    "citation": Workload("citation", 100_000_000, 16.0, 1, 100_000, False, torch.int64, 128,
                         torch.float16, 1.0, 8192, [15, 10, 5]),
    # scaled-down variants for CPU-side tests and quick GPU parity runs
    "mini_social": Workload("mini_social", 4_000, 120.0, 1, 1_500, True, torch.int32, 602,
                            torch.float32, 1.0, 64, [25, 10]),
    "mini_copurchase": Workload("mini_copurchase", 30_000, 30.0, 1, 3_000, True, torch.int32, 100,
                                torch.float32, 0.2, 256, [15, 10, 5], bias_rates=[1.0, 4.0]),
    "mini_citation": Workload("mini_citation", 50_000, 16.0, 1, 5_000, False, torch.int64, 128,
                              torch.float16, 1.0, 256, [15, 10, 5]),
}

# config 4: sweep on the co-purchase graph
SWEEP_BATCHES = [256, 1024, 4096, 16384]
SWEEP_CACHE_FRACS = [0.05, 0.2, 0.5, 1.0]
SWEEP_BIAS_RATES = [1.0, 2.0, 4.0, 8.0]


def get_config(name: str) -> Workload:
    return CONFIGS[name]
