"""Feature tables, the degree-ranked cache split and seed batches (harness code)."""
from dataclasses import dataclass
from typing import Optional

import math
import numpy as np
import torch

from .graphs import Graph, hash_stream, _lsr


def make_features(num_nodes: int, dim: int, dtype=torch.float32, feat_seed: int = 0,
                  device="cpu", rows_per_chunk: int = 1 << 22) -> torch.Tensor:
    """i.i.d. N(0,1) rows.  Values never affect timing; they make copies checkable."""
    g = torch.Generator(device=device)
    g.manual_seed(0x5EED0000 + feat_seed)
    out = torch.empty((num_nodes, dim), dtype=dtype, device=device)
    for r0 in range(0, num_nodes, rows_per_chunk):
        r1 = min(num_nodes, r0 + rows_per_chunk)
        out[r0:r1] = torch.randn((r1 - r0, dim), generator=g, device=device, dtype=torch.float32).to(dtype)
    return out


def padded_rows(n_rows: int, dim: int, dtype, device="cpu", row_align: int = 0,
                pin_memory: bool = False) -> torch.Tensor:
    """An [n_rows, dim] tensor whose rows start row_align bytes apart or a multiple of it
    (row_align = 0: packed).  It is a column slice of a wider buffer, so rows are dense but
    separated by padding; 128 gives every row whole cache lines."""
    elem = torch.empty(0, dtype=dtype).element_size()
    wide = dim
    if row_align:
        assert row_align % elem == 0
        wide = (dim * elem + row_align - 1) // row_align * row_align // elem
    buf = torch.zeros((n_rows, wide), dtype=dtype, device=device, pin_memory=pin_memory)
    return buf[:, :dim] if wide != dim else buf


@dataclass
class CacheSplit:
    cache_map: torch.Tensor            # int32 [N]: c >= 0 -> row c of feat_dev; c < 0 -> row -c-1 of feat_host
    feat_dev: Optional[torch.Tensor]   # [n_cached, dim] on the compute device (None if n_cached == 0)
    feat_host: Optional[torch.Tensor]  # [N - n_cached, dim] in (pinned) host memory (None if empty)
    n_cached: int


def degree_ranked_cache(graph: Graph, full: Optional[torch.Tensor], frac: float,
                        pin_host: bool = False, row_align: int = 0) -> CacheSplit:
    """Static cache of the hottest rows, hotness = degree (the policy the paper cites from
    PaGraph in Sec. II-B and uses, as the nodes accessed most often, in its ablation).
    Rank nodes by (degree descending, id ascending); the first ceil(frac * N) ranks live in
    the device cache at slot = rank, the others in the host store at slot = rank - n_cached.
    row_align > 0 pads the rows of both stores (see padded_rows)."""
    N = graph.num_nodes
    n_cached = min(N, int(math.ceil(frac * N)))
    deg = graph.degrees()
    order = torch.sort(deg, descending=True, stable=True).indices
    rank = torch.empty(N, dtype=torch.int64, device=deg.device)
    rank[order] = torch.arange(N, dtype=torch.int64, device=deg.device)
    cache_map = torch.where(rank < n_cached, rank, -(rank - n_cached) - 1).to(torch.int32)
    feat_dev = feat_host = None
    if full is not None:
        order_f = order.to(full.device)
        if n_cached > 0:
            if row_align:
                feat_dev = padded_rows(n_cached, full.shape[1], full.dtype, full.device, row_align)
                step = 1 << 20
                for r0 in range(0, n_cached, step):
                    r1 = min(n_cached, r0 + step)
                    feat_dev[r0:r1] = full[order_f[r0:r1]]
            else:
                feat_dev = full[order_f[:n_cached]].contiguous()
        if n_cached < N:
            rest = order_f[n_cached:]
            host = padded_rows(N - n_cached, full.shape[1], full.dtype, "cpu", row_align, pin_memory=pin_host)
            step = 1 << 20
            for r0 in range(0, N - n_cached, step):
                r1 = min(N - n_cached, r0 + step)
                host[r0:r1] = full[rest[r0:r1]].cpu()
            feat_host = host
    return CacheSplit(cache_map, feat_dev, feat_host, n_cached)


def seed_batch(num_nodes: int, num_seeds: int, base_seed: int, batch: int, dtype=np.int32) -> np.ndarray:
    """num_seeds distinct node ids, uniform, in draw order; independent of the sampler's stream."""
    assert num_seeds <= num_nodes
    got = np.zeros(0, dtype=np.int64)
    rnd = 0
    while got.shape[0] < num_seeds:
        j = torch.arange(rnd * 4 * num_seeds, (rnd + 1) * 4 * num_seeds, dtype=torch.int64)
        cand = (_lsr(hash_stream(base_seed, 1000 + batch, j), 1) % num_nodes).numpy()
        allc = np.concatenate([got, cand])
        _, first = np.unique(allc, return_index=True)
        got = allc[np.sort(first)]
        rnd += 1
    return got[:num_seeds].astype(dtype)
