"""The multi-threaded host sampler ("Sampling Device = CPU, Workers = n") against the oracle:
identical arrays for every hop, whatever the number of worker threads."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_07421_amd as a3
from helpers import blocks_equal, check_block_invariants
from workloads import get_config, make_graph, degree_ranked_cache, seed_batch

Q = 65536
_graphs = {}


def _graph(name):
    if name not in _graphs:
        w = get_config(name)
        g = make_graph(w.num_nodes, w.mean_degree, w.d_min, w.d_max, w.a, w.symmetric, w.graph_seed,
                       w.idx_dtype)
        _graphs[name] = (w, g, g.indptr.numpy(), g.indices.numpy())
    return _graphs[name]


@pytest.mark.parametrize("name", ["tiny", "mini_social", "mini_copurchase", "mini_citation"])
def test_cpu_sampler_matches_oracle(name):
    w, g, ip, ix = _graph(name)
    cm = degree_ranked_cache(g, None, 0.3).cache_map.numpy()
    s3 = a3.CpuSampler(3)
    batch = min(w.batch, 64)
    for gamma in (1.0, 4.0):
        for b in range(2):
            seeds = seed_batch(w.num_nodes, batch, 0, b, dtype=ix.dtype)
            got = s3.sample_blocks(ip, ix, seeds, w.fanouts, cm, int(gamma * Q), b)
            want = oracle.sample_blocks(ip, ix, seeds, w.fanouts, cm, int(gamma * Q), b)
            blocks_equal(got, want)
            if b == 0:
                check_block_invariants(ip, ix, seeds, w.fanouts, got)
    s3.close()


def test_vector_forms_of_the_draws_agree_with_the_scalar_form():
    differ, forms = a3.check_vector_forms()
    assert differ == 0
    print(f"vector forms checked on this CPU: {forms}")


@pytest.mark.parametrize("form", [1, 2, 3])
def test_cpu_sampler_matches_oracle_in_every_vector_form(form):
    """the whole sampler with its draws forced to the scalar, AVX2 and AVX-512 forms; rows longer
    than one group of 64 slots, row ends inside a group, both weight classes"""
    if not a3.set_vector_form(form):
        pytest.skip("this CPU lacks the form")
    try:
        w, g, ip, ix = _graph("mini_social")
        cm = degree_ranked_cache(g, None, 0.3).cache_map.numpy()
        s2 = a3.CpuSampler(2)
        for gamma, fan in ((1.0, w.fanouts), (4.0, w.fanouts), (1.0, [31, 2]), (8.0, [1, 40])):
            seeds = seed_batch(w.num_nodes, 48, 0, 5, dtype=ix.dtype)
            got = s2.sample_blocks(ip, ix, seeds, fan, cm, int(gamma * Q), 11)
            want = oracle.sample_blocks(ip, ix, seeds, fan, cm, int(gamma * Q), 11)
            blocks_equal(got, want)
        s2.close()
    finally:
        assert a3.set_vector_form(0)


@pytest.mark.parametrize("percent", [1, 30, 60, 10000])
def test_one_class_scan_with_too_few_and_too_many_survivors(percent):
    """a first bar that far too few draws clear (the second scan takes over: always at 1 %, for
    part of the rows at 30 and 60 %), and one that everything clears"""
    assert not a3.set_first_bar_percent(0)
    assert a3.set_first_bar_percent(percent)
    try:
        w, g, ip, ix = _graph("mini_social")
        s2 = a3.CpuSampler(2)
        for fan in ([25, 10], [1, 3], [64]):
            seeds = seed_batch(w.num_nodes, 64, 2, 7, dtype=ix.dtype)
            blocks_equal(s2.sample_blocks(ip, ix, seeds, fan, None, Q, 3),
                         oracle.sample_blocks(ip, ix, seeds, fan, None, Q, 3))
        s2.close()
    finally:
        assert a3.set_first_bar_percent(100)


def test_result_does_not_depend_on_the_number_of_workers():
    w, g, ip, ix = _graph("mini_social")
    cm = degree_ranked_cache(g, None, 0.5).cache_map.numpy()
    seeds = seed_batch(w.num_nodes, 64, 1, 0, dtype=ix.dtype)
    ref = None
    for n in (1, 2, 8, 0):
        s = a3.CpuSampler(n)
        assert s.n_workers >= 1
        got = s.sample_blocks(ip, ix, seeds, [25, 10], cm, 8 * Q, 5)
        again = s.sample_blocks(ip, ix, seeds, [25, 10], cm, 8 * Q, 5)   # the sampler cleans up after itself
        blocks_equal(got, again)
        if ref is None:
            ref = got
            blocks_equal(got, oracle.sample_blocks(ip, ix, seeds, [25, 10], cm, 8 * Q, 5))
        else:
            blocks_equal(got, ref)
        s.close()


@pytest.mark.parametrize("gamma", [1.5, 64.0, 65535.0])
def test_weight_classes_and_shapes(gamma):
    w, g, ip, ix = _graph("mini_social")
    s = a3.CpuSampler(4)
    for frac in (0.05, 0.5, 1.0):
        cm = degree_ranked_cache(g, None, frac).cache_map.numpy()
        for n_seeds, fan in [(1, [5]), (7, [70]), (50, [1, 1, 1, 1]), (33, [70, 3, 2, 1])]:
            seeds = seed_batch(w.num_nodes, n_seeds, 3, n_seeds, dtype=ix.dtype)
            blocks_equal(s.sample_blocks(ip, ix, seeds, fan, cm, int(gamma * Q), 9),
                         oracle.sample_blocks(ip, ix, seeds, fan, cm, int(gamma * Q), 9))
    s.close()


def test_errors_and_edge_cases():
    w, g, ip, ix = _graph("tiny")
    s = a3.CpuSampler(2)
    empty = s.sample_blocks(ip, ix, np.zeros(0, dtype=ix.dtype), [3, 2])
    assert empty.n_dst == [0, 0] and empty.n_edges == [0, 0] and empty.input_nodes.shape[0] == 0
    for bad in ([5, 9, 5], [5, w.num_nodes], [-1]):
        with pytest.raises(a3.A3Error) as ei:
            s.sample_blocks(ip, ix, np.array(bad, dtype=ix.dtype), [2])
        assert ei.value.code == -4
    with pytest.raises(a3.A3Error) as ei:
        s.sample_blocks(ip, ix, np.array([1], dtype=ix.dtype), [2], None, 1)
    assert ei.value.code == -1
    seeds = seed_batch(w.num_nodes, 40, 3, 1, dtype=ix.dtype)   # still works, map left clean
    blocks_equal(s.sample_blocks(ip, ix, seeds, [4, 3]), oracle.sample_blocks(ip, ix, seeds, [4, 3]))
    # isolated nodes
    indptr = np.array([0, 0, 1, 2, 2], dtype=np.int64)
    indices = np.array([2, 1], dtype=np.int64)
    seeds = np.array([0, 1, 3], dtype=np.int64)
    blocks_equal(s.sample_blocks(indptr, indices, seeds, [4, 4]), oracle.sample_blocks(indptr, indices, seeds, [4, 4]))
    s.close()
