"""GPU parity of the block mean aggregation against the oracle (fp64).

Tolerance, derived from the arithmetic: the kernel adds d fp32 values in edge order (d - 1
roundings of relative size u = 2^-24 on partial sums bounded by S = sum |x|), divides by d (one
more rounding) and, for half output, rounds once to binary16 (relative 2^-11):
    |got - want| <= (d + 1) * u * S / d                      float32
    |got - want| <= (d + 1) * u * S / d + 2^-11 * |want| + 2^-25  float16 (2^-25: half subnormal step / 2)
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_07421_amd as a3
from helpers import blocks_equal
from workloads import get_config, make_graph, make_features, degree_ranked_cache, seed_batch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
U32 = 2.0 ** -24


def _bound(indptr, indices, x, want, half):
    absx = np.abs(x.astype(np.float64))
    S = oracle.block_mean(indptr, indices, absx.astype(np.float32))  # mean |x| = S / d
    d = np.diff(indptr).astype(np.float64)[:, None]
    tol = (d + 1) * U32 * S * 1.0000001  # S/d already taken by the mean
    if half:
        tol = tol + 2.0 ** -11 * np.abs(want) + 2.0 ** -25
    return tol


def _check(ctx, indptr, indices, x_np, tag):
    print(f"[case] block_mean {tag} n_dst={len(indptr) - 1} n_src={x_np.shape[0]} dim={x_np.shape[1]} "
          f"dtype={x_np.dtype}", flush=True)
    want = oracle.block_mean(indptr, indices, x_np)
    got = ctx.block_mean(torch.from_numpy(indptr).to(DEV), torch.from_numpy(indices).to(DEV),
                         torch.from_numpy(x_np).to(DEV))
    got = got.cpu().numpy().astype(np.float64)
    tol = _bound(indptr, indices, x_np, want, x_np.dtype == np.float16)
    err = np.abs(got - want)
    assert np.all(err <= tol), f"{tag}: max excess {np.max(err - tol)}"
    return got


def _random_block(rng, n_dst, n_src, max_deg):
    deg = rng.integers(0, max_deg + 1, size=n_dst)
    indptr = np.zeros(n_dst + 1, dtype=np.int32)
    indptr[1:] = np.cumsum(deg)
    indices = rng.integers(0, n_src, size=int(indptr[-1])).astype(np.int32)
    return indptr, indices


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("dim", [1, 2, 3, 7, 8, 64, 100, 128, 301, 602, 1030, 4104])
def test_block_mean_matches_oracle_over_row_widths(dtype, dim):
    """every vector width (dim odd, = 2 mod 4, = 4 mod 8, ...), every lanes-per-row and
    vectors-per-lane count, and rows wider than one column tile"""
    rng = np.random.default_rng(dim)
    ctx = a3.Context(8, [2])
    n_dst, n_src = (300, 517) if dim <= 1030 else (40, 61)
    indptr, indices = _random_block(rng, n_dst, n_src, 13)
    x = (rng.standard_normal((n_src, dim)) * 3).astype(dtype)
    got = _check(ctx, indptr, indices, x, "widths")
    deg = np.diff(indptr)
    assert np.all(got[deg == 0] == 0.0)
    ctx.close()


def test_block_mean_edge_cases():
    rng = np.random.default_rng(0)
    ctx = a3.Context(8, [2])
    # no destinations; destinations without edges only; one destination with 1024 edges
    out = ctx.block_mean(torch.zeros(1, dtype=torch.int32, device=DEV),
                         torch.zeros(0, dtype=torch.int32, device=DEV),
                         torch.ones((4, 6), dtype=torch.float32, device=DEV))
    assert out.shape == (0, 6)
    x = rng.standard_normal((9, 10)).astype(np.float32)
    _check(ctx, np.zeros(6, dtype=np.int32), np.zeros(0, dtype=np.int32), x, "no edges")
    ip = np.array([0, 1024], dtype=np.int32)
    _check(ctx, ip, rng.integers(0, 9, size=1024).astype(np.int32), x, "one long row")
    # unaligned views: rows start at odd element offsets -> narrowest vector path
    base = torch.from_numpy(rng.standard_normal(1 + 50 * 6).astype(np.float32)).to(DEV)
    xv = base[1:].view(50, 6)
    indptr, indices = _random_block(rng, 20, 50, 5)
    got = ctx.block_mean(torch.from_numpy(indptr).to(DEV), torch.from_numpy(indices).to(DEV), xv)
    want = oracle.block_mean(indptr, indices, xv.cpu().numpy())
    np.testing.assert_allclose(got.cpu().numpy(), want, rtol=1e-6, atol=1e-6)
    # indices outside the source list are skipped, never dereferenced
    bad = np.array([0, 1, 99, -5], dtype=np.int32)
    got = ctx.block_mean(torch.tensor([0, 4], dtype=torch.int32, device=DEV),
                         torch.from_numpy(bad).to(DEV), torch.from_numpy(x).to(DEV)).cpu().numpy()
    np.testing.assert_allclose(got[0], (x[0] + x[1]) / 4, rtol=1e-6)
    with pytest.raises(a3.A3Error):
        lib = a3.lib()
        rc = lib.a3_block_mean(ctx._h, None, None, 1, 1, None, 7, 4, None)
        ctx._check(rc)
    ctx.close()


@pytest.mark.parametrize("name", ["mini_social", "mini_copurchase", "mini_citation"])
def test_block_mean_on_sampled_blocks(name):
    """the step after the path: aggregate the gathered rows over the outermost block, and a
    hidden layer's rows over the inner blocks, with the counts taken on the device"""
    w = get_config(name)
    g = make_graph(w.num_nodes, w.mean_degree, w.d_min, w.d_max, w.a, w.symmetric, w.graph_seed,
                   w.idx_dtype)
    full = make_features(w.num_nodes, w.feat_dim, w.feat_dtype)
    split = degree_ranked_cache(g, full, w.cache_frac, pin_host=True)
    d_ip, d_ix, d_cm = g.indptr.to(DEV), g.indices.to(DEV), split.cache_map.to(DEV)
    fd = split.feat_dev.to(DEV)
    seeds = seed_batch(w.num_nodes, w.batch, 0, 3, dtype=g.indices.numpy().dtype)
    ctx = a3.Context(w.batch, w.fanouts)
    H = len(w.fanouts)
    rows = torch.zeros((min(w.num_nodes, 200_000), w.feat_dim), dtype=w.feat_dtype, device=DEV)
    agg = torch.full_like(rows, 7.0)
    ctx.sample_blocks_begin(d_ip, d_ix, torch.from_numpy(seeds).to(DEV), w.fanouts, d_cm, 65536, 3)
    ctx.gather_input_features(fd, split.feat_host, d_cm, rows)
    ctx.block_mean_of_hop(H - 1, rows, agg)           # queued before the host knows any count
    blk = ctx.sample_blocks_end()
    torch.cuda.synchronize()
    # the oracle's own chain: its blocks, its rows, its means (nothing of the GPU's feeds it)
    ob = oracle.sample_blocks(g.indptr.numpy(), g.indices.numpy(), seeds, w.fanouts,
                              split.cache_map.numpy(), 65536, 3)
    blocks_equal(blk.to_host(), ob)
    x_np = oracle.gather_features(split.feat_dev.numpy(),
                                  None if split.feat_host is None else split.feat_host.numpy(),
                                  split.cache_map.numpy(), ob.input_nodes)
    want = oracle.block_mean(ob.blk_indptr[-1], ob.blk_indices[-1], x_np)
    got = agg[: blk.n_dst[-1]].cpu().numpy().astype(np.float64)
    tol = _bound(ob.blk_indptr[-1], ob.blk_indices[-1], x_np, want, x_np.dtype == np.float16)
    assert np.all(np.abs(got - want) <= tol)
    assert torch.all(agg[blk.n_dst[-1]:] == 7.0)      # rows past n_dst are not written
    # inner blocks through the explicit entry point
    for h in range(H - 1):
        _check(ctx, ob.blk_indptr[h], ob.blk_indices[h], x_np[: ob.n_src[h]], f"{name} hop {h}")
    ctx.close()
