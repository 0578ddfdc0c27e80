"""GPU parity of the padded-row forms: the retrieve, the block mean and a pipeline with stores and
outputs whose rows start a multiple of 16 / 128 bytes apart.  The payload must equal the oracle's
(which knows nothing of padding); padding bytes of the outputs are unspecified."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_07421_amd as a3
from helpers import blocks_equal
from workloads import (get_config, make_graph, make_features, degree_ranked_cache, padded_rows,
                       seed_batch)

pytestmark = pytest.mark.gpu
Q = 65536
DEV = "cuda:0"


@pytest.fixture(scope="module")
def world():
    w = get_config("mini_copurchase")
    g = make_graph(w.num_nodes, w.mean_degree, w.d_min, w.d_max, w.a, w.symmetric, w.graph_seed,
                   w.idx_dtype)
    return w, g


@pytest.mark.parametrize("dim,dtype,align", [(602, torch.float32, 128), (602, torch.float32, 16),
                                             (100, torch.float32, 128), (33, torch.float16, 16),
                                             (33, torch.float16, 2), (5, torch.float32, 8),
                                             (1030, torch.float16, 128), (7, torch.float16, 128)])
def test_strided_gather_matches_oracle(world, dim, dtype, align):
    w, g = world
    full = make_features(g.num_nodes, dim, dtype, feat_seed=3)
    ctx = a3.Context(16, [2])
    for frac in (1.0, 0.3, 0.0):
        split = degree_ranked_cache(g, full, frac, pin_host=True, row_align=align)
        packed = degree_ranked_cache(g, full, frac)
        d_cm = split.cache_map.to(DEV)
        d_fd = None
        if split.feat_dev is not None:
            d_fd = padded_rows(split.n_cached, dim, dtype, DEV, align)
            d_fd.copy_(split.feat_dev)
            assert d_fd.shape[0] < 2 or d_fd.stride(0) * d_fd.element_size() % align == 0
        for n_ids in (1, 777, 4000):
            print(f"[case] strided gather dim={dim} {dtype} align={align} frac={frac} n_ids={n_ids}", flush=True)
            ids = seed_batch(g.num_nodes, n_ids, 4, n_ids, dtype=np.int32)
            want = oracle.gather_features(None if packed.feat_dev is None else packed.feat_dev.numpy(),
                                          None if packed.feat_host is None else packed.feat_host.numpy(),
                                          packed.cache_map.numpy(), ids)
            # padded stores into a padded output, and into a packed one
            out_p = padded_rows(n_ids, dim, dtype, DEV, align)
            ctx.gather_features(d_fd, split.feat_host, d_cm, torch.from_numpy(ids).to(DEV), out=out_p)
            got = ctx.gather_features(d_fd, split.feat_host, d_cm, torch.from_numpy(ids).to(DEV))
            torch.cuda.synchronize()
            assert out_p.cpu().numpy().tobytes() == want.tobytes()
            assert got.cpu().numpy().tobytes() == want.tobytes()
    ctx.close()


@pytest.mark.parametrize("dim,dtype,align", [(602, torch.float32, 128), (100, torch.float32, 16),
                                             (33, torch.float16, 16), (128, torch.float16, 128)])
def test_strided_block_mean_and_device_count_path(world, dim, dtype, align):
    w, g = world
    full = make_features(g.num_nodes, dim, dtype, feat_seed=4)
    split = degree_ranked_cache(g, full, 1.0, row_align=align)
    d_ip, d_ix, d_cm = g.indptr.to(DEV), g.indices.to(DEV), split.cache_map.to(DEV)
    d_fd = padded_rows(split.n_cached, dim, dtype, DEV, align)
    d_fd.copy_(split.feat_dev)
    ctx = a3.Context(64, w.fanouts)
    seeds = seed_batch(w.num_nodes, 64, 0, 5, dtype=np.int32)
    rows = padded_rows(20000, dim, dtype, DEV, align)
    agg = padded_rows(20000, dim, dtype, DEV, align)
    H = len(w.fanouts)
    ctx.sample_blocks_begin(d_ip, d_ix, torch.from_numpy(seeds).to(DEV), w.fanouts, d_cm, Q, 5)
    ctx.gather_input_features(d_fd, None, d_cm, rows)
    ctx.block_mean_of_hop(H - 1, rows, agg)
    blk = ctx.sample_blocks_end()
    torch.cuda.synchronize()
    # the oracle's own chain (packed rows; it knows nothing of padding)
    ob = oracle.sample_blocks(g.indptr.numpy(), g.indices.numpy(), seeds, w.fanouts,
                              split.cache_map.numpy(), Q, 5)
    blocks_equal(blk.to_host(), ob)
    n_in, n_dst = ob.n_src[-1], ob.n_dst[-1]
    x_np = oracle.gather_features(np.ascontiguousarray(split.feat_dev.numpy()), None,
                                  split.cache_map.numpy(), ob.input_nodes)
    assert rows[:n_in].cpu().numpy().tobytes() == x_np.tobytes()
    want = oracle.block_mean(ob.blk_indptr[-1], ob.blk_indices[-1], x_np)
    got = agg[:n_dst].cpu().numpy().astype(np.float64)
    mean_abs = oracle.block_mean(ob.blk_indptr[-1], ob.blk_indices[-1], np.abs(x_np.astype(np.float32)))
    d = np.diff(ob.blk_indptr[-1]).astype(np.float64)[:, None]
    tol = (d + 1) * 2.0 ** -24 * mean_abs * 1.0000001
    if dtype == torch.float16:
        tol = tol + 2.0 ** -11 * np.abs(want) + 2.0 ** -25
    assert np.all(np.abs(got - want) <= tol)
    # explicit entry point: padded x into a packed result
    got2 = ctx.block_mean(blk.blk_indptr[0], blk.blk_indices[0], rows[: blk.n_src[0]])
    want2 = oracle.block_mean(ob.blk_indptr[0], ob.blk_indices[0], x_np[: ob.n_src[0]])
    np.testing.assert_allclose(got2.cpu().numpy().astype(np.float64), want2, rtol=2e-3, atol=2e-3)
    ctx.close()


def test_pipeline_with_padded_rows(world):
    w, g = world
    full = make_features(g.num_nodes, 30, torch.float32, feat_seed=6)
    split = degree_ranked_cache(g, full, 0.3, pin_host=True, row_align=128)
    d_ip, d_ix, d_cm = g.indptr.to(DEV), g.indices.to(DEV), split.cache_map.to(DEV)
    d_fd = padded_rows(split.n_cached, 30, torch.float32, DEV, 128)
    d_fd.copy_(split.feat_dev)
    pipe = a3.Pipeline(a3.A3_PIPE_MODE2, 2, 128, w.fanouts)
    outs = [padded_rows(w.num_nodes, 30, torch.float32, DEV, 128) for _ in range(2)]
    seeds = [seed_batch(w.num_nodes, 100, 0, b, dtype=np.int32) for b in range(4)]
    d_seeds = [torch.from_numpy(s).to(DEV) for s in seeds]
    torch.cuda.synchronize()
    for b in range(2):
        pipe.submit(d_ip, d_ix, d_seeds[b], w.fanouts, d_cm, 4 * Q, b, d_fd, split.feat_host, outs[b])
    for b in range(4):
        blk = pipe.wait()
        ob = oracle.sample_blocks(g.indptr.numpy(), g.indices.numpy(), seeds[b], w.fanouts,
                                  split.cache_map.numpy(), 4 * Q, b)
        blocks_equal(blk.to_host(), ob)
        got = outs[b % 2][: blk.n_src[-1]].cpu()
        assert torch.equal(got, full[torch.from_numpy(ob.input_nodes).long()])
        if b + 2 < 4:
            pipe.submit(d_ip, d_ix, d_seeds[b + 2], w.fanouts, d_cm, 4 * Q, b + 2, d_fd, split.feat_host,
                        outs[b % 2])
    pipe.close()
