"""Pins for the oracle's multi-hop sampling + reindex and its feature gather."""
import numpy as np
import pytest
import torch

import oracle
from helpers import check_block_invariants, blocks_equal
from workloads import get_config, make_graph, make_features, degree_ranked_cache, seed_batch

Q = 65536


def _graph(name):
    w = get_config(name)
    g = make_graph(w.num_nodes, w.mean_degree, w.d_min, w.d_max, w.a, w.symmetric, w.graph_seed,
                   w.idx_dtype)
    return w, g


@pytest.fixture(scope="module")
def tiny():
    return _graph("tiny")


def test_generated_graph_is_simple_and_sorted(tiny):
    w, g = tiny
    ip, ix = g.indptr.numpy(), g.indices.numpy()
    assert ip[0] == 0 and ip[-1] == ix.shape[0] and np.all(np.diff(ip) >= 0)
    rows = np.repeat(np.arange(g.num_nodes), np.diff(ip))
    assert np.all(ix != rows), "no self loops"
    same = rows[1:] == rows[:-1]
    assert np.all(ix[1:][same] > ix[:-1][same]), "rows sorted, no repeated neighbour"
    key = rows.astype(np.int64) * g.num_nodes + ix
    rev = ix.astype(np.int64) * g.num_nodes + rows
    assert np.array_equal(np.sort(key), np.sort(rev)), "undirected"


def test_hand_built_graph_brute_force():
    """A 6-node graph small enough to follow by hand.  fanout 2 per hop."""
    #   0: 1 2 3 4     1: 0 2      2: 0 1      3: 0      4: 0 5      5: 4
    rows = [[1, 2, 3, 4], [0, 2], [0, 1], [0], [0, 5], [4]]
    indptr = np.cumsum([0] + [len(r) for r in rows]).astype(np.int64)
    indices = np.concatenate(rows).astype(np.int32)
    seeds = np.array([3, 0], dtype=np.int32)
    b = oracle.sample_blocks(indptr, indices, seeds, [2, 2], rng_seed=4)
    check_block_invariants(indptr, indices, seeds, [2, 2], b)
    # hop 0: node 3 has one neighbour (0, already local id 1); node 0 keeps 2 of its 4
    pick0 = oracle.select(4, 0, 0, 4, 2)
    assert list(b.blk_indptr[0]) == [0, 1, 3]
    assert b.blk_indices[0][0] == 1
    assert list(b.blk_eids[0]) == [int(indptr[3])] + [0 + s for s in pick0]
    new = [rows[0][s] for s in pick0]                       # both new: 3 and 0 are the only known ids
    new = [v for v in new if v not in (3, 0)]
    assert list(b.input_nodes[:2 + len(new)]) == [3, 0] + new
    assert list(b.blk_indices[0][1:]) == [[3, 0].index(v) if v in (3, 0) else 2 + new.index(v)
                                          for v in (rows[0][s] for s in pick0)]
    # hop 1 is driven by D_1 = S_0 and replays hop 0's choice for node 0 only if the hop
    # number were ignored; it must not be
    assert b.n_dst[1] == b.n_src[0]


def test_invariants_on_all_small_workloads():
    for name in ["tiny", "mini_social", "mini_copurchase", "mini_citation"]:
        w, g = _graph(name)
        ip, ix = g.indptr.numpy(), g.indices.numpy()
        cache = degree_ranked_cache(g, None, w.cache_frac)
        cm = cache.cache_map.numpy()
        for gamma in w.bias_rates:
            for batch in range(2):
                seeds = seed_batch(w.num_nodes, w.batch, 0, batch, dtype=ix.dtype)
                b = oracle.sample_blocks(ip, ix, seeds, w.fanouts, cm, int(gamma * Q), rng_seed=batch)
                check_block_invariants(ip, ix, seeds, w.fanouts, b)


def test_same_seed_same_result_different_seed_differs(tiny):
    w, g = tiny
    ip, ix = g.indptr.numpy(), g.indices.numpy()
    seeds = seed_batch(w.num_nodes, w.batch, 0, 0)
    a = oracle.sample_blocks(ip, ix, seeds, w.fanouts, rng_seed=0)
    b = oracle.sample_blocks(ip, ix, seeds, w.fanouts, rng_seed=0)
    blocks_equal(a, b)
    c = oracle.sample_blocks(ip, ix, seeds, w.fanouts, rng_seed=1)
    assert not np.array_equal(a.blk_eids[0], c.blk_eids[0])


def test_uniform_cases_ignore_the_device_map(tiny):
    """gamma = 1, or a cache holding everything or nothing, is plain uniform sampling."""
    w, g = tiny
    ip, ix = g.indptr.numpy(), g.indices.numpy()
    seeds = seed_batch(w.num_nodes, w.batch, 0, 3)
    base = oracle.sample_blocks(ip, ix, seeds, w.fanouts, None, Q, rng_seed=3)
    part = degree_ranked_cache(g, None, 0.3).cache_map.numpy()
    full = degree_ranked_cache(g, None, 1.0).cache_map.numpy()
    none = degree_ranked_cache(g, None, 0.0).cache_map.numpy()
    assert (full >= 0).all() and (none < 0).all()
    blocks_equal(base, oracle.sample_blocks(ip, ix, seeds, w.fanouts, part, Q, rng_seed=3))
    blocks_equal(base, oracle.sample_blocks(ip, ix, seeds, w.fanouts, full, 8 * Q, rng_seed=3))
    blocks_equal(base, oracle.sample_blocks(ip, ix, seeds, w.fanouts, none, 8 * Q, rng_seed=3))
    biased = oracle.sample_blocks(ip, ix, seeds, w.fanouts, part, 8 * Q, rng_seed=3)
    assert not np.array_equal(base.blk_eids[0], biased.blk_eids[0])


def test_bias_raises_hit_rate_and_shrinks_the_input_set():
    """Sec. II-B / III-A: favouring cached nodes raises the cache hit rate and lets reindex
    drop more duplicates (fewer input nodes)."""
    w, g = _graph("mini_copurchase")
    ip, ix = g.indptr.numpy(), g.indices.numpy()
    cm = degree_ranked_cache(g, None, 0.2).cache_map.numpy()
    hit, n_in = [], []
    for gamma in [1, 2, 4, 8]:
        hs, ns = 0.0, 0
        for batch in range(4):
            seeds = seed_batch(w.num_nodes, w.batch, 0, batch)
            b = oracle.sample_blocks(ip, ix, seeds, w.fanouts, cm, gamma * Q, rng_seed=batch)
            hs += float((cm[b.input_nodes] >= 0).mean())
            ns += b.input_nodes.shape[0]
        hit.append(hs / 4)
        n_in.append(ns / 4)
    assert all(a < b for a, b in zip(hit, hit[1:])), hit
    assert all(a > b for a, b in zip(n_in, n_in[1:])), n_in


def test_edge_cases():
    w, g = _graph("tiny")
    ip, ix = g.indptr.numpy(), g.indices.numpy()
    empty = oracle.sample_blocks(ip, ix, np.zeros(0, dtype=np.int32), [3, 2])
    assert empty.n_dst == [0, 0] and empty.n_edges == [0, 0] and empty.input_nodes.shape[0] == 0
    # isolated node: appears as destination and source, no edges
    ip2 = np.array([0, 0, 1, 2], dtype=np.int64)
    ix2 = np.array([2, 1], dtype=np.int64)
    b = oracle.sample_blocks(ip2, ix2, np.array([0, 1], dtype=np.int64), [4])
    assert b.n_edges == [1] and list(b.blk_indptr[0]) == [0, 0, 1] and list(b.input_nodes) == [0, 1, 2]
    with pytest.raises(ValueError):
        oracle.sample_blocks(ip, ix, np.array([1], dtype=np.int32), [0])
    with pytest.raises(ValueError):
        oracle.sample_blocks(ip, ix, np.array([1], dtype=np.int32), [2], bias_q16=1000)
    with pytest.raises(ValueError):
        oracle.sample_blocks(ip, ix, np.array([w.num_nodes], dtype=np.int32), [2])


def test_gather_equals_library_index_select():
    w, g = _graph("tiny")
    for dtype, dim in [(torch.float32, 64), (torch.float16, 128), (torch.float32, 602), (torch.float32, 100)]:
        full = make_features(g.num_nodes, dim, dtype, feat_seed=1)
        for frac in [1.0, 0.2, 0.0]:
            split = degree_ranked_cache(g, full, frac)
            cm = split.cache_map
            # each node lives in exactly one store, at the slot the map names
            n_c = split.n_cached
            assert int((cm >= 0).sum()) == n_c and n_c == int(np.ceil(frac * g.num_nodes))
            if n_c:
                ids_c = torch.nonzero(cm >= 0).flatten()
                assert torch.equal(split.feat_dev[cm[ids_c].long()], full[ids_c])
                assert torch.unique(cm[ids_c]).shape[0] == n_c
            if n_c < g.num_nodes:
                ids_h = torch.nonzero(cm < 0).flatten()
                assert torch.equal(split.feat_host[(-cm[ids_h].long() - 1)], full[ids_h])
            ids = seed_batch(g.num_nodes, 777, 5, 0, dtype=np.int64)
            fd = None if split.feat_dev is None else split.feat_dev.numpy()
            fh = None if split.feat_host is None else split.feat_host.numpy()
            out = oracle.gather_features(fd, fh, cm.numpy(), ids)
            expect = torch.index_select(full, 0, torch.from_numpy(ids)).numpy()
            assert out.tobytes() == expect.tobytes()
            out32 = oracle.gather_features(fd, fh, cm.numpy(), ids.astype(np.int32))
            assert out32.tobytes() == expect.tobytes()
    # no map: identity into the device store
    out = oracle.gather_features(full.numpy(), None, None, ids)
    assert out.tobytes() == torch.index_select(full, 0, torch.from_numpy(ids)).numpy().tobytes()
    assert oracle.gather_features(full.numpy(), None, None, np.zeros(0, dtype=np.int64)).shape == (0, 100)
