"""Power-law synthetic graphs in CSR form (harness code, not part of the method).

The paper evaluates on OGB datasets, Reddit, Yelp and Amazon (Sec. IV-A);
none of them is available here, so graphs of the same published shape (node
count, edge count, skewed degrees) stand in for them.  Degrees follow a
continuous Pareto law floored to integers; neighbours are drawn proportionally
to the target degree (Chung-Lu style), so hubs are popular neighbours too.
Rows are sorted, without self-loops or repeated neighbours.
"""
from dataclasses import dataclass

import torch

_MASK64 = (1 << 64) - 1


def _s64(c: int) -> int:
    c &= _MASK64
    return c - (1 << 64) if c >= (1 << 63) else c


_GOLD = _s64(0x9E3779B97F4A7C15)
_C1 = _s64(0xBF58476D1CE4E5B9)
_C2 = _s64(0x94D049BB133111EB)


def _lsr(z: torch.Tensor, k: int) -> torch.Tensor:
    """logical shift right of an int64 tensor"""
    return (z >> k) & ((1 << (64 - k)) - 1)


def mix64(z: torch.Tensor) -> torch.Tensor:
    """SplitMix64 finaliser on int64 tensors (wrapping arithmetic)."""
    z = z + _GOLD
    z = (z ^ _lsr(z, 30)) * _C1
    z = (z ^ _lsr(z, 27)) * _C2
    return z ^ _lsr(z, 31)


def hash_stream(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """64 hashed bits per element of idx, a different sequence per (seed, stream)."""
    base = _s64((seed * 0xD1342543DE82EF95 + stream * 0xA0761D6478BD642F + 0x1234567) & _MASK64)
    return mix64(mix64(idx + base) ^ _s64(0x2545F4914F6CDD1D * (stream + 1)))


def uniform01(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """float64 in [0, 1)"""
    return _lsr(hash_stream(seed, stream, idx), 11).to(torch.float64) * (2.0 ** -53)


def powerlaw_degrees(num_nodes: int, mean: float, d_min: int, d_max: int, a: float,
                     graph_seed: int, device="cpu") -> torch.Tensor:
    """d_v = clip(floor(x_min * (1 - r_v)^(-1/(a-1))), d_min, d_max); x_min bisected to the mean."""
    idx = torch.arange(num_nodes, dtype=torch.int64, device=device)
    r = uniform01(graph_seed, 1, idx)
    shape = (1.0 - r).pow(-1.0 / (a - 1.0))

    def degrees(x_min):
        return torch.clamp(torch.floor(x_min * shape), d_min, d_max)

    lo, hi = 1e-3, float(d_max)
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        if degrees(mid).mean().item() < mean:
            lo = mid
        else:
            hi = mid
    return degrees(hi).to(torch.int64)


@dataclass
class Graph:
    indptr: torch.Tensor    # int64 [N+1]
    indices: torch.Tensor   # int32 or int64 [nnz]
    num_nodes: int

    @property
    def nnz(self) -> int:
        return int(self.indices.shape[0])

    def degrees(self) -> torch.Tensor:
        return self.indptr[1:] - self.indptr[:-1]

    def stats(self) -> dict:
        d = self.degrees()
        return {"num_nodes": self.num_nodes, "nnz": self.nnz,
                "mean_degree": float(d.double().mean().item()) if self.num_nodes else 0.0,
                "max_degree": int(d.max().item()) if self.num_nodes else 0,
                "idx_bytes": self.indices.element_size()}


def _draw_targets(cum: torch.Tensor, total: int, graph_seed: int, edge_ids: torch.Tensor):
    r = _lsr(hash_stream(graph_seed, 2, edge_ids), 1) % total
    return torch.searchsorted(cum, r, right=True)


def chung_lu_csr(target_deg: torch.Tensor, symmetric: bool, graph_seed: int,
                 idx_dtype=torch.int32, chunk_edges: int = 1 << 26) -> Graph:
    """CSR graph whose row v has about target_deg[v] sorted, distinct neighbours != v."""
    device = target_deg.device
    N = int(target_deg.shape[0])
    out_k = (target_deg + 1) // 2 if symmetric else target_deg
    cum = torch.cumsum(target_deg, 0)
    total = int(cum[-1].item())
    start = torch.zeros(N + 1, dtype=torch.int64, device=device)
    start[1:] = torch.cumsum(out_k, 0)
    n_draws = int(start[-1].item())
    bounds = [0]
    # split nodes into ranges of at most chunk_edges draws
    starts_cpu = start.cpu()
    while bounds[-1] < N:
        lo = bounds[-1]
        limit = int(starts_cpu[lo].item()) + chunk_edges
        hi = int(torch.searchsorted(starts_cpu, torch.tensor(limit), right=True).item()) - 1
        bounds.append(min(N, max(hi, lo + 1)))
    key_chunks, count_chunks, dst_chunks = [], [], []
    for lo, hi in zip(bounds[:-1], bounds[1:]):
        e0, e1 = int(starts_cpu[lo].item()), int(starts_cpu[hi].item())
        eid = torch.arange(e0, e1, dtype=torch.int64, device=device)
        src = torch.searchsorted(start, eid, right=True) - 1
        dst = _draw_targets(cum, total, graph_seed, eid)
        keep = src != dst
        src, dst = src[keep], dst[keep]
        if symmetric:
            key_chunks.append(src * N + dst)
            key_chunks.append(dst * N + src)
        else:
            key = torch.unique((src - lo) * N + dst)       # sorted, distinct
            rows = key // N
            count_chunks.append(torch.bincount(rows, minlength=hi - lo))
            dst_chunks.append((key - rows * N).to(idx_dtype))
        del eid, src, dst, keep
    if symmetric:
        key = torch.unique(torch.cat(key_chunks)) if key_chunks else torch.zeros(0, dtype=torch.int64, device=device)
        del key_chunks
        rows = key // N
        counts = torch.bincount(rows, minlength=N)
        indices = (key - rows * N).to(idx_dtype)
    else:
        counts = torch.cat(count_chunks) if count_chunks else torch.zeros(N, dtype=torch.int64, device=device)
        indices = torch.cat(dst_chunks) if dst_chunks else torch.zeros(0, dtype=idx_dtype, device=device)
    indptr = torch.zeros(N + 1, dtype=torch.int64, device=device)
    indptr[1:] = torch.cumsum(counts, 0)
    assert n_draws >= 0
    return Graph(indptr, indices, N)


def make_graph(num_nodes: int, mean_degree: float, d_min: int, d_max: int, a: float = 2.1,
               symmetric: bool = True, graph_seed: int = 0, idx_dtype=torch.int32,
               device="cpu") -> Graph:
    deg = powerlaw_degrees(num_nodes, mean_degree, d_min, d_max, a, graph_seed, device)
    return chung_lu_csr(deg, symmetric, graph_seed, idx_dtype)
