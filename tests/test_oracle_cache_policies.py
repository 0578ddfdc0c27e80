"""Pins for the oracle's cache policies: access counting, the static fill ranked by access count,
and the FIFO dynamic cache."""
import collections

import numpy as np
import pytest
import torch

import oracle
from workloads import make_graph, degree_ranked_cache


def test_count_accesses_is_a_histogram():
    rng = np.random.default_rng(0)
    counts = np.zeros(50, dtype=np.uint32)
    total = np.zeros(50, dtype=np.int64)
    for dtype in (np.int32, np.int64):
        ids = rng.integers(0, 50, size=300).astype(dtype)
        oracle.count_accesses(ids, counts)
        total += np.bincount(ids, minlength=50)
    assert np.array_equal(counts.astype(np.int64), total)
    with pytest.raises(ValueError):
        oracle.count_accesses(np.array([50], dtype=np.int32), counts)


def test_rank_cache_against_lexsort_and_invariants():
    rng = np.random.default_rng(1)
    n, n_cached = 1000, 137
    counts = rng.integers(0, 6, size=n).astype(np.uint32)     # many ties
    cache_map, order = oracle.rank_cache(counts, n_cached)
    want_order = np.lexsort((np.arange(n), -counts.astype(np.int64)))  # count desc, then id asc
    assert np.array_equal(order, want_order)
    rank = np.empty(n, dtype=np.int64)
    rank[want_order] = np.arange(n)
    assert np.array_equal(cache_map, np.where(rank < n_cached, rank, -(rank - n_cached) - 1))
    # each node in exactly one store, slots are bijections onto [0, n_cached) and [0, n - n_cached)
    dev = cache_map[cache_map >= 0]
    host = -cache_map[cache_map < 0] - 1
    assert sorted(dev) == list(range(n_cached)) and sorted(host) == list(range(n - n_cached))
    # nothing uncached was accessed more often than something cached
    assert counts[cache_map >= 0].min() >= counts[cache_map < 0].max()
    # edge cases: nothing cached, everything cached
    cm0, _ = oracle.rank_cache(counts, 0)
    assert np.all(cm0 < 0)
    cm1, _ = oracle.rank_cache(counts, n)
    assert np.all(cm1 >= 0)


def test_rank_cache_with_degrees_equals_the_generators_degree_ranked_split():
    g = make_graph(3000, 12.0, 1, 400, 2.1, True, 3, torch.int32)
    deg = g.degrees().numpy().astype(np.uint32)
    for frac in (0.0, 0.2, 1.0):
        split = degree_ranked_cache(g, None, frac)
        cache_map, _ = oracle.rank_cache(deg, split.n_cached)
        assert np.array_equal(cache_map, split.cache_map.numpy())


def _queue_simulation(n_nodes, n_slots, batches, rows_of):
    """FIFO cache told differently: a deque of cached nodes and a dict node -> slot."""
    q = collections.deque()
    slot_of = {}
    next_slot = 0
    feat = np.zeros((n_slots, rows_of(0).shape[0]), dtype=np.float32)
    for ids in batches:
        missed = [int(v) for v in ids if int(v) not in slot_of]  # judged as the batch arrives
        for v in missed:
            if len(q) == n_slots:
                old = q.popleft()
                s = slot_of.pop(old)
            else:
                s = next_slot
                next_slot += 1
            q.append(v)
            slot_of[v] = s
            feat[s] = rows_of(v)
    cache_map = np.array([slot_of.get(v, -v - 1) for v in range(n_nodes)], dtype=np.int32)
    return cache_map, feat


@pytest.mark.parametrize("n_slots,batch_len", [(16, 5), (16, 16), (7, 40), (1, 3)])
def test_fifo_cache_against_a_queue_simulation(n_slots, batch_len):
    """includes mini-batches with more misses than slots (early arrivals leave again at once)"""
    rng = np.random.default_rng(n_slots * 100 + batch_len)
    n_nodes, dim = 60, 3
    full = rng.standard_normal((n_nodes, dim)).astype(np.float32)
    batches = [rng.choice(n_nodes, size=batch_len, replace=False).astype(np.int32) for _ in range(12)]
    cache_map = (-np.arange(n_nodes) - 1).astype(np.int32)
    owner = np.full(n_slots, -1, dtype=np.int32)
    head = np.zeros(1, dtype=np.int32)
    feat = np.zeros((n_slots, dim), dtype=np.float32)
    for ids in batches:
        hits_before = int((cache_map[ids] >= 0).sum())
        m = oracle.cache_fifo_update(cache_map, owner, head, feat, ids, full[ids])
        assert m == len(ids) - hits_before
        assert 0 <= head[0] < n_slots
        # map and owners describe the same cache; cached rows hold the node's features
        for s in range(n_slots):
            if owner[s] >= 0:
                assert cache_map[owner[s]] == s and np.array_equal(feat[s], full[owner[s]])
        cached = np.flatnonzero(cache_map >= 0)
        assert len(cached) == (owner >= 0).sum() <= n_slots
        assert np.array_equal(cache_map[cache_map < 0], -np.flatnonzero(cache_map < 0) - 1)
    want_map, want_feat = _queue_simulation(n_nodes, n_slots, batches, lambda v: full[v])
    assert np.array_equal(cache_map, want_map)
    filled = owner >= 0
    assert np.array_equal(feat[filled], want_feat[filled])


def test_fifo_cache_hand_followed():
    # 3 slots; nodes 0..5; rows = [v, 10 v]
    full = np.array([[v, 10 * v] for v in range(6)], dtype=np.float32)
    cache_map = (-np.arange(6) - 1).astype(np.int32)
    owner = np.full(3, -1, dtype=np.int32)
    head = np.zeros(1, dtype=np.int32)
    feat = np.zeros((3, 2), dtype=np.float32)
    ids = np.array([4, 1], dtype=np.int32)
    assert oracle.cache_fifo_update(cache_map, owner, head, feat, ids, full[ids]) == 2
    assert list(owner) == [4, 1, -1] and head[0] == 2 and list(cache_map) == [-1, 1, -3, -4, 0, -6]
    ids = np.array([1, 5, 0], dtype=np.int32)       # 1 hits; 5 takes slot 2; 0 evicts 4 from slot 0
    assert oracle.cache_fifo_update(cache_map, owner, head, feat, ids, full[ids]) == 2
    assert list(owner) == [0, 1, 5] and head[0] == 1 and list(cache_map) == [0, 1, -3, -4, -5, 2]
    assert np.array_equal(feat, full[[0, 1, 5]])
