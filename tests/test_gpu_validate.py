"""a3_validate_graph / a3_validate_cache_map: valid inputs pass, each kind of planted mistake is
named.  The mistakes are planted in host copies of valid inputs; the kernels read nothing outside
the array sizes they are given, whatever the arrays hold."""
import numpy as np
import pytest
import torch

import paper_2511_07421_amd as a3
from workloads import get_config, make_graph, degree_ranked_cache

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _graph(name):
    w = get_config(name)
    g = make_graph(w.num_nodes, w.mean_degree, w.d_min, w.d_max, w.a, w.symmetric, w.graph_seed, w.idx_dtype)
    return w, g


def _expect(ctx, ip, ix, word):
    print(f"[case] validate_graph expects '{word}'", flush=True)
    with pytest.raises(a3.A3Error) as ei:
        ctx.validate_graph(torch.from_numpy(ip).to(DEV), torch.from_numpy(ix).to(DEV))
    assert ei.value.code == a3.A3_ERR_INPUT and word in str(ei.value), str(ei.value)


@pytest.mark.parametrize("name", ["tiny", "mini_social", "mini_copurchase", "mini_citation"])
def test_valid_graphs_and_maps_pass(name):
    w, g = _graph(name)
    ctx = a3.Context(8, [2])
    ctx.validate_graph(g.indptr.to(DEV), g.indices.to(DEV))
    for frac in (0.0, 0.3, 1.0):
        split = degree_ranked_cache(g, None, frac)
        ctx.validate_cache_map(split.cache_map.to(DEV), split.n_cached, w.num_nodes - split.n_cached)
    # an empty graph, and a graph without edges
    ctx.validate_graph(torch.zeros(1, dtype=torch.int64, device=DEV), torch.zeros(0, dtype=torch.int32, device=DEV))
    ctx.validate_graph(torch.zeros(5, dtype=torch.int64, device=DEV), torch.zeros(0, dtype=torch.int64, device=DEV))
    ctx.validate_cache_map(torch.zeros(0, dtype=torch.int32, device=DEV), 0, 0)
    ctx.close()


@pytest.mark.parametrize("name", ["mini_social", "mini_citation"])
def test_planted_mistakes_in_the_graph_are_named(name):
    w, g = _graph(name)
    ip0, ix0 = g.indptr.numpy(), g.indices.numpy()
    N, nnz = w.num_nodes, ix0.shape[0]
    deg = np.diff(ip0)
    v = int(np.argmax(deg >= 3))                       # a node with at least three neighbours
    lo = int(ip0[v])
    ctx = a3.Context(8, [2])
    # a row out of order; a neighbour twice
    ix = ix0.copy(); ix[lo], ix[lo + 1] = ix0[lo + 1], ix0[lo]
    _expect(ctx, ip0, ix, "strictly increasing")
    ix = ix0.copy(); ix[lo + 1] = ix0[lo]
    _expect(ctx, ip0, ix, "strictly increasing")
    # ids outside the graph, at the very end of indices and in the middle
    for bad in (N, -1):
        ix = ix0.copy(); ix[nnz - 1] = bad
        _expect(ctx, ip0, ix, "outside [0, num_nodes)")
    ix = ix0.copy(); ix[lo + 2] = N + 7
    _expect(ctx, ip0, ix, "outside [0, num_nodes)")
    # row bounds: decreasing inside the range, beyond nnz, negative
    u = int(np.argmax(deg[1:] >= 2)) + 1               # a node other than 0 with a row of its own
    ip = ip0.copy(); ip[u] = ip0[u + 1] + 1 if ip0[u + 1] + 1 <= nnz else ip0[u + 1]
    if ip[u] > ip[u + 1]:
        _expect(ctx, ip, ix0, "indptr decreases")
    ip = ip0.copy(); ip[u] = nnz + 5
    _expect(ctx, ip, ix0, "indptr decreases")
    ip = ip0.copy(); ip[u] = -3
    _expect(ctx, ip, ix0, "indptr decreases")
    # the ends
    ip = ip0.copy(); ip[N] = nnz - 1
    _expect(ctx, ip, ix0, "indptr[0] is not 0 or indptr[num_nodes] is not nnz")
    if deg[0] >= 1:
        ip = ip0.copy(); ip[0] = 1
        _expect(ctx, ip, ix0, "indptr[0] is not 0")
    # the untouched inputs still pass
    ctx.validate_graph(g.indptr.to(DEV), g.indices.to(DEV))
    ctx.close()


def test_planted_mistakes_in_the_device_map_are_named():
    w, g = _graph("mini_copurchase")
    split = degree_ranked_cache(g, None, 0.25)
    cm0 = split.cache_map.numpy()
    n_dev, n_host = split.n_cached, w.num_nodes - split.n_cached
    ctx = a3.Context(8, [2])

    def expect(cm, nd, nh, word):
        print(f"[case] validate_cache_map expects '{word}'", flush=True)
        with pytest.raises(a3.A3Error) as ei:
            ctx.validate_cache_map(torch.from_numpy(cm).to(DEV), nd, nh)
        assert ei.value.code == a3.A3_ERR_INPUT and word in str(ei.value), str(ei.value)

    cached = int(np.argmax(cm0 >= 0)); uncached = int(np.argmax(cm0 < 0))
    cm = cm0.copy(); cm[cached] = n_dev
    expect(cm, n_dev, n_host, "outside its store")
    cm = cm0.copy(); cm[uncached] = -n_host - 1
    expect(cm, n_dev, n_host, "outside its store")
    expect(cm0, n_dev - 1, n_host, "outside its store")         # a store smaller than the map says
    expect(cm0, n_dev, n_host - 1, "outside its store")
    other = int(np.flatnonzero(cm0 >= 0)[5])
    cm = cm0.copy(); cm[other] = cm0[cached]
    expect(cm, n_dev, n_host, "share a row")
    other = int(np.flatnonzero(cm0 < 0)[7])
    cm = cm0.copy(); cm[other] = cm0[uncached]
    expect(cm, n_dev, n_host, "share a row")
    cm = np.full_like(cm0, np.iinfo(np.int32).min); cm[0] = np.iinfo(np.int32).max
    expect(cm, n_dev, n_host, "outside its store")
    ctx.validate_cache_map(split.cache_map.to(DEV), n_dev, n_host)
    ctx.validate_cache_map(split.cache_map.to(DEV), n_dev + 9, n_host + 9)   # stores may be larger
    ctx.close()
