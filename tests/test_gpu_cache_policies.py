"""GPU parity of the cache policies: access counting and the static fill ranked by access count
(bit-exact), and a FIFO dynamic cache that evolves over several mini-batches while locality-aware
sampling reads it (map, owners, ring head and cached rows equal to the oracle's after every
mini-batch; the feedback between policy and sampler is part of what is compared)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_07421_amd as a3
from helpers import blocks_equal
from workloads import get_config, make_graph, make_features, seed_batch

pytestmark = pytest.mark.gpu
Q = 65536
DEV = "cuda:0"


@pytest.fixture(scope="module")
def world():
    w = get_config("mini_copurchase")
    g = make_graph(w.num_nodes, w.mean_degree, w.d_min, w.d_max, w.a, w.symmetric, w.graph_seed,
                   w.idx_dtype)
    full = make_features(w.num_nodes, 10, torch.float32)
    return w, g, full


def test_access_counts_and_ranked_fill_match_oracle(world):
    w, g, full = world
    d_ip, d_ix = g.indptr.to(DEV), g.indices.to(DEV)
    ctx = a3.Context(w.batch, w.fanouts)
    counts = torch.zeros(w.num_nodes, dtype=torch.int32, device=DEV)
    want = np.zeros(w.num_nodes, dtype=np.uint32)
    for b in range(5):   # pre-sampling: uniform, nothing cached yet
        seeds = seed_batch(w.num_nodes, w.batch, 7, b, dtype=np.int32)
        ctx.sample_blocks_begin(d_ip, d_ix, torch.from_numpy(seeds).to(DEV), w.fanouts, None, Q, b)
        ctx.cache_count_accesses(counts)           # queued before the host knows the count
        blk = ctx.sample_blocks_end()
        ob = oracle.sample_blocks(g.indptr.numpy(), g.indices.numpy(), seeds, w.fanouts, None, Q, b)
        oracle.count_accesses(ob.input_nodes.astype(np.int32), want)
    extra = torch.tensor([5, 5, 9, w.num_nodes - 1], dtype=torch.int64, device=DEV)   # explicit ids, repeated
    ctx.cache_count_accesses(counts, extra)
    oracle.count_accesses(extra.cpu().numpy(), want)
    assert np.array_equal(counts.cpu().numpy().view(np.uint32), want)
    assert want.max() >= 3 and (want == 0).any()
    for n_cached in (0, 1, w.num_nodes // 5, w.num_nodes):
        cm, order = ctx.cache_rank(counts, n_cached)
        want_cm, want_order = oracle.rank_cache(want, n_cached)
        assert np.array_equal(cm.cpu().numpy(), want_cm)
        assert np.array_equal(order.cpu().numpy(), want_order)
    # the stores of the fill are gathers along `order`; sampling + gather through them equals the
    # oracle run on the same map
    n_cached = w.num_nodes // 5
    cm, order = ctx.cache_rank(counts, n_cached)
    d_full = full.to(DEV)
    feat_dev = ctx.gather_features(d_full, None, None, order[:n_cached].contiguous())
    feat_host = ctx.gather_features(d_full, None, None, order[n_cached:].contiguous()).cpu().pin_memory()
    seeds = seed_batch(w.num_nodes, w.batch, 7, 99, dtype=np.int32)
    blk = ctx.sample_blocks(d_ip, d_ix, torch.from_numpy(seeds).to(DEV), w.fanouts, cm, 4 * Q, 99)
    rows = ctx.gather_features(feat_dev, feat_host, cm, blk.input_nodes)
    assert torch.equal(rows.cpu(), full[blk.input_nodes.cpu().long()])
    ob = oracle.sample_blocks(g.indptr.numpy(), g.indices.numpy(), seeds, w.fanouts,
                              oracle.rank_cache(want, n_cached)[0], 4 * Q, 99)
    blocks_equal(blk.to_host(), ob)
    ctx.close()


@pytest.mark.parametrize("n_slots,batch", [(3000, 128), (200, 256), (1, 16)])
def test_fifo_cache_evolves_like_the_oracle(world, n_slots, batch):
    """n_slots = 200 with ~10^4 input nodes per mini-batch: far more misses than slots"""
    w, g, full = world
    N, dim = w.num_nodes, full.shape[1]
    d_ip, d_ix = g.indptr.to(DEV), g.indices.to(DEV)
    host_store = full.clone().pin_memory()          # every row: uncached v reads row v
    ctx = a3.Context(batch, w.fanouts)
    cm = (-torch.arange(N, dtype=torch.int32) - 1).to(DEV)
    owner = torch.full((n_slots,), -1, dtype=torch.int32, device=DEV)
    state = torch.zeros(4, dtype=torch.int32, device=DEV)
    cache = torch.zeros((n_slots, dim), dtype=torch.float32, device=DEV)
    rows = torch.zeros((N, dim), dtype=torch.float32, device=DEV)
    o_cm = (-np.arange(N) - 1).astype(np.int32)
    o_owner = np.full(n_slots, -1, dtype=np.int32)
    o_head = np.zeros(1, dtype=np.int32)
    o_cache = np.zeros((n_slots, dim), dtype=np.float32)
    hit_rates = []
    for b in range(6):
        print(f"[case] fifo n_slots={n_slots} batch={batch} step={b}", flush=True)
        seeds = seed_batch(N, batch, 11, b, dtype=np.int32)
        ctx.sample_blocks_begin(d_ip, d_ix, torch.from_numpy(seeds).to(DEV), w.fanouts, cm, 4 * Q, b)
        ctx.gather_input_features(cache, host_store, cm, rows)
        ctx.cache_fifo_update(cm, owner, state, cache, rows)     # all queued, no host wait
        blk = ctx.sample_blocks_end()
        ob = oracle.sample_blocks(g.indptr.numpy(), g.indices.numpy(), seeds, w.fanouts, o_cm, 4 * Q, b)
        blocks_equal(blk.to_host(), ob)                        # the sampler saw the same cache
        o_rows = oracle.gather_features(o_cache, full.numpy(), o_cm, ob.input_nodes.astype(np.int32))
        hit_rates.append(float((o_cm[ob.input_nodes] >= 0).mean()))
        misses = oracle.cache_fifo_update(o_cm, o_owner, o_head, o_cache, ob.input_nodes.astype(np.int32), o_rows)
        torch.cuda.synchronize()
        n_in = blk.n_src[-1]
        assert rows[:n_in].cpu().numpy().tobytes() == o_rows.tobytes()
        st = state.cpu().numpy()
        assert st[0] == o_head[0] and st[1] == misses
        assert np.array_equal(cm.cpu().numpy(), o_cm)
        assert np.array_equal(owner.cpu().numpy(), o_owner)
        filled = o_owner >= 0
        assert np.array_equal(cache.cpu().numpy()[filled], o_cache[filled])
    if n_slots == 3000:
        assert hit_rates[0] == 0.0 and hit_rates[-1] > 0.05   # the cache warms up
    ctx.close()


def test_fifo_update_with_explicit_ids_and_int64(world):
    w, g, full = world
    N, dim, n_slots = 500, 6, 40
    rng = np.random.default_rng(5)
    table = rng.standard_normal((N, dim)).astype(np.float16)
    ctx = a3.Context(8, [2])
    cm = (-torch.arange(N, dtype=torch.int32) - 1).to(DEV)
    owner = torch.full((n_slots,), -1, dtype=torch.int32, device=DEV)
    state = torch.zeros(4, dtype=torch.int32, device=DEV)
    cache = torch.zeros((n_slots, dim), dtype=torch.float16, device=DEV)
    o_cm, o_owner = cm.cpu().numpy().copy(), owner.cpu().numpy().copy()
    o_head, o_cache = np.zeros(1, dtype=np.int32), np.zeros((n_slots, dim), dtype=np.float16)
    for b, n_ids in enumerate([0, 1, 39, 41, 3000 % N, 64]):
        ids = rng.choice(N, size=n_ids, replace=False).astype(np.int64)
        d_ids = torch.from_numpy(ids).to(DEV)
        d_rows = torch.from_numpy(table[ids]).to(DEV)
        ctx.cache_fifo_update(cm, owner, state, cache, d_rows, d_ids)
        oracle.cache_fifo_update(o_cm, o_owner, o_head, o_cache, ids, table[ids])
        torch.cuda.synchronize()
        assert np.array_equal(cm.cpu().numpy(), o_cm) and np.array_equal(owner.cpu().numpy(), o_owner)
        assert state.cpu().numpy()[0] == o_head[0]
        filled = o_owner >= 0
        assert cache.cpu().numpy()[filled].tobytes() == o_cache[filled].tobytes()
    ctx.close()
