"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle.
Bit-exact on every index array; byte-exact on gathered rows (they are copies)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_07421_amd as a3
from helpers import blocks_equal, check_block_invariants
from workloads import get_config, make_graph, make_features, degree_ranked_cache, seed_batch

pytestmark = pytest.mark.gpu
Q = 65536
DEV = "cuda:0"
_graphs = {}


def _graph(name):
    if name not in _graphs:
        w = get_config(name)
        g = make_graph(w.num_nodes, w.mean_degree, w.d_min, w.d_max, w.a, w.symmetric, w.graph_seed,
                       w.idx_dtype)
        _graphs[name] = (w, g, g.indptr.to(DEV), g.indices.to(DEV))
    return _graphs[name]


def _compare(ctx, w, g, d_indptr, d_indices, seeds, fanouts, cm_host, gamma, rng_seed, tag=""):
    print(f"[case] {tag} graph={w.name} seeds={len(seeds)} fanouts={fanouts} gamma={gamma} "
          f"rng_seed={rng_seed}", flush=True)
    d_seeds = torch.from_numpy(seeds).to(DEV)
    d_cm = None if cm_host is None else torch.from_numpy(cm_host).to(DEV)
    got = ctx.sample_blocks(d_indptr, d_indices, d_seeds, fanouts, d_cm, int(gamma * Q), rng_seed)
    got = got.to_host()
    want = oracle.sample_blocks(g.indptr.numpy(), g.indices.numpy(), seeds, fanouts, cm_host,
                                int(gamma * Q), rng_seed)
    blocks_equal(got, want)
    return got


@pytest.mark.parametrize("name", ["tiny", "mini_social", "mini_copurchase", "mini_citation"])
def test_sample_blocks_matches_oracle(name):
    w, g, d_ip, d_ix = _graph(name)
    ctx = a3.Context(w.batch, w.fanouts)
    cm = degree_ranked_cache(g, None, w.cache_frac).cache_map.numpy()
    n_batches = 8 if name == "tiny" else 2
    for gamma in w.bias_rates:
        for b in range(n_batches):
            seeds = seed_batch(w.num_nodes, w.batch, 0, b, dtype=g.indices.numpy().dtype)
            got = _compare(ctx, w, g, d_ip, d_ix, seeds, w.fanouts, cm, gamma, b, "main")
            if b == 0:
                check_block_invariants(g.indptr.numpy(), g.indices.numpy(), seeds, w.fanouts, got)
    ctx.close()


@pytest.mark.parametrize("gamma", [1.5, 2.0, 8.0, 64.0, 65535.0])
def test_weighted_selection_matches_oracle(gamma):
    """partial cache: both weight classes present; large gamma floods the challenger buffer"""
    w, g, d_ip, d_ix = _graph("mini_social")
    ctx = a3.Context(128, [25, 10])
    for frac in [0.05, 0.5]:
        cm = degree_ranked_cache(g, None, frac).cache_map.numpy()
        seeds = seed_batch(w.num_nodes, 100, 1, 0)
        _compare(ctx, w, g, d_ip, d_ix, seeds, [25, 10], cm, gamma, 11, f"frac={frac}")
    ctx.close()


def _hub_graph():
    """wide rows and hubs; seeds: the largest rows, middling ones and the smallest"""
    if "hubs" not in _graphs:
        g = make_graph(20_000, 700.0, 40, 12_000, 2.1, True, 5, torch.int32)
        deg = (g.indptr[1:] - g.indptr[:-1]).numpy()
        assert deg.max() > 4096 and (deg > 64).sum() > 1000
        order = np.argsort(-deg, kind="stable")
        seeds = np.concatenate([order[:24], order[2000:2040], order[-16:]]).astype(np.int32)
        _graphs["hubs"] = (get_config("mini_social"), g, g.indptr.to(DEV), g.indices.to(DEV), seeds)
    return _graphs["hubs"]


def test_too_few_draws_above_the_threshold_take_one_more_scan():
    """About one node in 10^5 keeps fewer candidates than its fanout and scans its row once more
    with a lower threshold.  With the testing flag the first threshold keeps about fanout / 2, so
    nearly every wide node and hub goes that way (and, weighted, through the second launch)."""
    w, g, d_ip, d_ix, seeds = _hub_graph()
    ctx = a3.Context(len(seeds), [15, 3], flags=a3.A3_TEST_FEW_DRAWS)
    for frac, gamma, fan in [(0.5, 1.0, [15, 3]), (0.5, 4.0, [15, 3]), (0.1, 2.0, [10, 3]), (0.9, 8.0, [5]),
                             (1.0, 4.0, [15, 2]), (0.3, 64.0, [15])]:
        cm = degree_ranked_cache(g, None, frac).cache_map.numpy()
        _compare(ctx, w, g, d_ip, d_ix, seeds, fan, cm, gamma, 31, f"few draws frac={frac}")
        assert ctx.sample_stats()["exhaustive_nodes"] <= 2
    ctx.close()
    w, g, d_ip, d_ix = _graph("mini_social")
    ctx = a3.Context(128, [25, 10], flags=a3.A3_TEST_FEW_DRAWS)
    cm = degree_ranked_cache(g, None, 0.3).cache_map.numpy()
    for b, gamma in enumerate([1.0, 1.5, 4.0]):
        _compare(ctx, w, g, d_ip, d_ix, seed_batch(w.num_nodes, 128, 1, b), [25, 10], cm, gamma, b, "few draws")
    ctx.close()


def test_weighted_candidate_lists_of_every_size():
    """Wide rows and hubs with many cached neighbours: the two candidate lists of the weighted
    path hold from a few to several hundred slots (every register count of the selection, and
    past its limit, where the row is scanned a second time instead)."""
    w, g, d_ip, d_ix, seeds = _hub_graph()
    ctx = a3.Context(len(seeds), [15, 3])
    for frac in [0.1, 0.5, 0.9]:
        cm = degree_ranked_cache(g, None, frac).cache_map.numpy()
        for gamma, fan in [(1.25, [15, 3]), (2.0, [15]), (3.0, [10, 3]), (4.0, [15, 2]), (6.0, [5, 3]),
                           (8.0, [15]), (12.0, [10]), (20.0, [15])]:
            _compare(ctx, w, g, d_ip, d_ix, seeds, fan, cm, gamma, 21, f"lists frac={frac}")
    ctx.close()


def test_malformed_row_lengths_are_refused_not_followed():
    """row starts that do not increase, or a row longer than 2^31-1: an error code, no sampling
    of that row (its neighbour slots would lie outside `indices`)"""
    indices = torch.arange(6, dtype=torch.int32, device=DEV) % 3
    ctx = a3.Context(4, [2])
    seeds = torch.tensor([0, 1, 2], dtype=torch.int32, device=DEV)
    # every row START below stays inside `indices` (6 entries); only a row's LENGTH is wrong:
    # row 1 of the first has length -2, row 2 of the second 2^32 + 5
    for indptr in ([0, 4, 2, 6], [0, 2, 4, (1 << 32) + 9]):
        with pytest.raises(a3.A3Error) as ei:
            ctx.sample_blocks(torch.tensor(indptr, dtype=torch.int64, device=DEV), indices, seeds, [2])
        assert ei.value.code == a3.A3_ERR_CAPACITY
    ok = ctx.sample_blocks(torch.tensor([0, 2, 4, 6], dtype=torch.int64, device=DEV), indices, seeds, [2])
    assert ok.n_edges == [6]
    ctx.close()


def test_one_weight_class_equals_uniform_sampling():
    """everything cached or nothing cached: gamma has no effect (Sec. III-A: equal weights are
    plain uniform sampling), on the oracle and on the GPU alike"""
    w, g, d_ip, d_ix = _graph("mini_social")
    ctx = a3.Context(128, [25, 10])
    seeds = seed_batch(w.num_nodes, 100, 1, 3)
    ref = _compare(ctx, w, g, d_ip, d_ix, seeds, [25, 10], None, 1.0, 4, "no map")
    for frac in (0.0, 1.0):
        cm = degree_ranked_cache(g, None, frac).cache_map.numpy()
        for gamma in (1.0, 4.0, 1000.0):
            got = _compare(ctx, w, g, d_ip, d_ix, seeds, [25, 10], cm, gamma, 4, f"one class frac={frac}")
            blocks_equal(got, ref)
    ctx.close()


def test_largest_fanouts():
    """fanouts up to the library's maximum (1024): candidate lists beyond the register paths,
    several chosen slots per lane, fewer wavefronts per workgroup for lack of LDS"""
    g = make_graph(20_000, 700.0, 40, 12_000, 2.1, True, 5, torch.int32)
    deg = (g.indptr[1:] - g.indptr[:-1]).numpy()
    d_ip, d_ix = g.indptr.to(DEV), g.indices.to(DEV)
    w = get_config("mini_social")
    order = np.argsort(-deg, kind="stable")
    seeds = np.concatenate([order[:6], order[3000:3006], order[-4:]]).astype(np.int32)
    cm = degree_ranked_cache(g, None, 0.5).cache_map.numpy()
    for fan in ([a3.A3_MAX_FANOUT], [200, 3], [65, 64], [500, 1]):
        ctx = a3.Context(len(seeds), fan)
        for gamma in (1.0, 4.0):
            _compare(ctx, w, g, d_ip, d_ix, seeds, fan, cm, gamma, 31, "large fanout")
        ctx.close()


def test_node_ids_above_two_to_the_32():
    """8-byte ids whose high word is not zero (it is part of the Philox counter): a graph of
    2^32 + 1000 nodes, all of them isolated except a thousand around the 2^32 boundary.  The CSR
    row starts are 34 GB on the device; on the host the array comes zero-mapped and the oracle
    touches only the frontier's entries."""
    free, _ = torch.cuda.mem_get_info()
    if free < 80 << 30:
        pytest.skip("needs 80 GB of free device memory")
    N = (1 << 32) + 1000
    lo = (1 << 32) - 500                     # nodes lo .. lo + 999 have neighbours, among themselves
    n_act, deg = 1000, 300
    rng = np.random.default_rng(9)
    rows = np.stack([np.sort(rng.choice(n_act, size=deg, replace=False)) for _ in range(n_act)]) + lo
    indices = rows.reshape(-1).astype(np.int64)
    ip_h = np.zeros(N + 1, dtype=np.int64)   # calloc: untouched pages cost nothing
    ip_h[lo:lo + n_act + 1] = np.arange(n_act + 1, dtype=np.int64) * deg
    ip_h[lo + n_act:] = n_act * deg
    d_ip = torch.zeros(N + 1, dtype=torch.int64, device=DEV)
    d_ip[lo:lo + n_act + 1] = torch.arange(n_act + 1, dtype=torch.int64, device=DEV) * deg
    d_ip[lo + n_act:] = n_act * deg
    d_ix = torch.from_numpy(indices).to(DEV)
    seeds = (lo + rng.choice(n_act, size=40, replace=False)).astype(np.int64)
    assert (seeds >= 1 << 32).any() and (seeds < 1 << 32).any()
    ctx = a3.Context(64, [10, 5])
    print(f"[case] ids above 2^32: N={N} seeds={len(seeds)}", flush=True)
    got = ctx.sample_blocks(d_ip, d_ix, torch.from_numpy(seeds).to(DEV), [10, 5], None, Q, 77).to_host()
    want = oracle.sample_blocks(ip_h, indices, seeds, [10, 5], None, Q, 77)
    blocks_equal(got, want)
    assert (got.input_nodes >= 1 << 32).any()
    # 4-byte ids cannot name these nodes: refused, not truncated
    with pytest.raises(a3.A3Error) as ei:
        ctx.sample_blocks(d_ip, torch.zeros(4, dtype=torch.int32, device=DEV),
                          torch.zeros(1, dtype=torch.int32, device=DEV), [2])
    assert ei.value.code == a3.A3_ERR_INVALID_ARG
    ctx.close()
    del d_ip
    torch.cuda.empty_cache()


def test_exhaustive_selection_path_matches_oracle():
    for name in ["tiny", "mini_copurchase"]:
        w, g, d_ip, d_ix = _graph(name)
        ctx = a3.Context(w.batch, w.fanouts, flags=a3.A3_FORCE_RADIX)
        cm = degree_ranked_cache(g, None, 0.2).cache_map.numpy()
        seeds = seed_batch(w.num_nodes, min(w.batch, 64), 2, 0)
        _compare(ctx, w, g, d_ip, d_ix, seeds, w.fanouts, cm, 1.0, 5, "radix uniform")
        _compare(ctx, w, g, d_ip, d_ix, seeds, w.fanouts, cm, 4.0, 5, "radix weighted")
        ctx.close()


def test_fanout_shapes_and_edge_cases():
    w, g, d_ip, d_ix = _graph("mini_social")
    ctx = a3.Context(300, [70, 3, 2, 1], flags=a3.A3_VALIDATE)
    cm = degree_ranked_cache(g, None, 0.3).cache_map.numpy()
    # empty batch
    empty = ctx.sample_blocks(d_ip, d_ix, torch.zeros(0, dtype=torch.int32, device=DEV), [3, 2])
    assert empty.n_dst == [0, 0] and empty.n_edges == [0, 0] and empty.input_nodes.numel() == 0
    # one seed; fanout above 64 (more than one candidate per lane); four hops; fanout 1
    for seeds_n, fan in [(1, [5]), (7, [70]), (300, [1, 1, 1, 1]), (33, [70, 3, 2, 1]), (257, [2, 2])]:
        seeds = seed_batch(w.num_nodes, seeds_n, 3, seeds_n)
        _compare(ctx, w, g, d_ip, d_ix, seeds, fan, cm, 1.0, 9, "shape")
        _compare(ctx, w, g, d_ip, d_ix, seeds, fan, cm, 3.0, 9, "shape weighted")
    # capacity and input errors come back as codes, and the context keeps working
    with pytest.raises(a3.A3Error) as ei:
        ctx.sample_blocks(d_ip, d_ix, torch.arange(301, dtype=torch.int32, device=DEV), [2])
    assert ei.value.code == a3.A3_ERR_CAPACITY
    with pytest.raises(a3.A3Error) as ei:
        ctx.sample_blocks(d_ip, d_ix, torch.tensor([5, 9, 5], dtype=torch.int32, device=DEV), [2])
    assert ei.value.code == a3.A3_ERR_INPUT
    with pytest.raises(a3.A3Error) as ei:
        ctx.sample_blocks(d_ip, d_ix, torch.tensor([5, w.num_nodes], dtype=torch.int32, device=DEV), [2])
    assert ei.value.code == a3.A3_ERR_INPUT
    seeds = seed_batch(w.num_nodes, 50, 3, 1)
    _compare(ctx, w, g, d_ip, d_ix, seeds, [4, 3], cm, 1.0, 1, "after errors")
    ctx.close()


def test_empty_batch_between_batches_on_a_plain_context():
    """no seeds, on a context without A3_VALIDATE and after a call that left a frontier behind:
    empty blocks, and the next call is unaffected"""
    w, g, d_ip, d_ix = _graph("mini_social")
    ctx = a3.Context(64, [5, 3])
    cm = degree_ranked_cache(g, None, 0.3).cache_map.numpy()
    seeds = seed_batch(w.num_nodes, 64, 3, 2)
    _compare(ctx, w, g, d_ip, d_ix, seeds, [5, 3], cm, 2.0, 5, "before the empty batch")
    for d_cm in (None, torch.from_numpy(cm).to(DEV)):
        empty = ctx.sample_blocks(d_ip, d_ix, torch.zeros(0, dtype=torch.int32, device=DEV), [5, 3], d_cm, 2 * Q, 6)
        assert empty.n_dst == [0, 0] and empty.n_src == [0, 0] and empty.n_edges == [0, 0]
        assert empty.input_nodes.numel() == 0
        assert [int(t[0].item()) for t in empty.blk_indptr] == [0, 0]
    seeds = seed_batch(w.num_nodes, 50, 3, 4)
    _compare(ctx, w, g, d_ip, d_ix, seeds, [5, 3], cm, 2.0, 7, "after the empty batch")
    _compare(ctx, w, g, d_ip, d_ix, seeds, [5, 3], None, 1.0, 8, "after the empty batch, no map")
    ctx.close()


@pytest.mark.parametrize("flags", [0, a3.A3_VALIDATE])
@pytest.mark.parametrize("host_workgroups", [0, 16])
def test_input_rows_by_stored_map_entries_and_by_lookup_agree(flags, host_workgroups):
    """The retrieve of a mini-batch's input nodes uses the device-map entries that the sampling call
    stored (same map given to both calls); given an equal map at another address, or a sampling
    call without a map, it looks every id up.  All three give the oracle's rows."""
    w, g, d_ip, d_ix = _graph("mini_copurchase")
    full = make_features(g.num_nodes, w.feat_dim, w.feat_dtype, feat_seed=6)
    split = degree_ranked_cache(g, full, 0.25, pin_host=True)
    d_cm, d_fd = split.cache_map.to(DEV), split.feat_dev.to(DEV)
    d_cm2 = d_cm.clone()
    ctx = a3.Context(w.batch, w.fanouts, flags=flags)
    ctx.set_gather_host_workgroups(host_workgroups)
    for b, gamma in enumerate((1.0, 4.0)):
        seeds = seed_batch(w.num_nodes, w.batch, 0, b)
        d_seeds = torch.from_numpy(seeds).to(DEV)
        want = oracle.sample_blocks(g.indptr.numpy(), g.indices.numpy(), seeds, w.fanouts,
                                    split.cache_map.numpy(), int(gamma * Q), b)
        want_rows = oracle.gather_features(split.feat_dev.numpy(), split.feat_host.numpy(),
                                           split.cache_map.numpy(), want.input_nodes)
        n = want.n_src[-1]
        for tag, sample_map, gather_map in (("stored entries", d_cm, d_cm), ("lookup, other address", d_cm, d_cm2),
                                            ("lookup, sampled without a map", None, d_cm)):
            if sample_map is None and gamma != 1.0:
                continue
            print(f"[case] input rows: {tag} gamma={gamma} flags={flags} host_workgroups={host_workgroups}", flush=True)
            out = torch.full((n + 3, w.feat_dim), 7.0, dtype=w.feat_dtype, device=DEV)
            ctx.sample_blocks_begin(d_ip, d_ix, d_seeds, w.fanouts, sample_map, int(gamma * Q), b)
            ctx.gather_input_features(d_fd, split.feat_host, gather_map, out)
            got = ctx.sample_blocks_end().to_host()
            torch.cuda.synchronize()
            blocks_equal(got, want)
            assert out[:n].cpu().numpy().tobytes() == want_rows.tobytes()
            assert bool((out[n:] == 7.0).all())
    ctx.close()


@pytest.mark.parametrize("flags", [a3.A3_TEST_MAP_RANGE, a3.A3_TEST_MAP_RANGE | a3.A3_VALIDATE])
def test_relabel_map_ranges_down_to_the_bottom_of_int32_and_refills(flags):
    """The relabel map is never cleaned: each call writes values below the previous call's.  With
    the testing flag the ranges start just above the bottom of int32 (negative values) and every
    third call refills the map; a run of calls with different seeds, fanouts and an input error in
    between must equal the oracle call by call."""
    w, g, d_ip, d_ix = _graph("mini_copurchase")
    cm = degree_ranked_cache(g, None, 0.3).cache_map.numpy()
    ctx = a3.Context(200, [15, 10, 5], flags=flags)
    for b in range(8):
        seeds = seed_batch(w.num_nodes, 200 - 20 * b, 5, b)
        fan = [[15, 10, 5], [3, 2], [15]][b % 3]
        _compare(ctx, w, g, d_ip, d_ix, seeds, fan, cm if b % 2 else None, 4.0 if b % 2 else 1.0, b, "map ranges")
        if b == 4 and (flags & a3.A3_VALIDATE):
            with pytest.raises(a3.A3Error):
                ctx.sample_blocks(d_ip, d_ix, torch.tensor([7, 9, 7], dtype=torch.int32, device=DEV), [2])
    ctx.close()


def test_weighted_launch_plan_follows_the_cache_and_keeps_the_blocks():
    """With few neighbours cached the first launch of a weighted hop decides almost no wide node;
    the context then runs its next 16 weighted calls with the single full launch per hop, tries
    the two-launch plan again, and stays with it once the cache holds enough.  The blocks equal
    the oracle's under either plan; calls without weights do not count."""
    w, g, d_ip, d_ix = _graph("mini_social")
    sparse = degree_ranked_cache(g, None, 0.01).cache_map.numpy()
    dense = degree_ranked_cache(g, None, 0.6).cache_map.numpy()
    ctx = a3.Context(64, [25, 10])
    plans = []
    for b in range(19):
        seeds = seed_batch(w.num_nodes, 64 - b, 3, b)
        _compare(ctx, w, g, d_ip, d_ix, seeds, [25, 10], sparse, 4.0, b, "launch plan")
        st = ctx.sample_stats()
        plans.append(st["launch_plan"])
        if st["launch_plan"] == 2:
            assert st["deferred_wide_nodes"] == 0 and st["deferred_hubs"] == 0
        if b == 5:
            _compare(ctx, w, g, d_ip, d_ix, seeds, [25, 10], None, 1.0, b, "launch plan, no weights")
            assert ctx.sample_stats()["launch_plan"] == 0
    assert plans == [1] + [2] * 16 + [1, 2]
    for b in range(19, 19 + 18):
        seeds = seed_batch(w.num_nodes, 64, 3, b)
        if b in (19, 35, 36):
            _compare(ctx, w, g, d_ip, d_ix, seeds, [25, 10], dense, 4.0, b, "launch plan, dense cache")
        else:
            d_cm = torch.from_numpy(dense).to(DEV)
            ctx.sample_blocks(d_ip, d_ix, torch.from_numpy(seeds).to(DEV), [25, 10], d_cm, 4 * Q, b)
        plans.append(ctx.sample_stats()["launch_plan"])
    assert plans[19:] == [2] * 15 + [1, 1, 1]
    ctx.close()


def test_reserve_before_the_first_call_changes_no_result():
    """a3_reserve makes the relabel map and the cached-node bitmap ahead of the first call (the
    pipeline test checks the bytes); a larger graph later enlarges them as before"""
    w, g, d_ip, d_ix = _graph("mini_copurchase")
    cm = degree_ranked_cache(g, None, 0.3).cache_map.numpy()
    ctx = a3.Context(64, [15, 10, 5])
    ctx.reserve(w.num_nodes)
    for b in range(3):
        _compare(ctx, w, g, d_ip, d_ix, seed_batch(w.num_nodes, 64, 9, b), [15, 10, 5], cm, 4.0, b, "reserved")
    ctx.reserve(10)                                               # smaller: nothing to do
    w2, g2, d_ip2, d_ix2 = _graph("mini_citation")                # larger graph on the same context
    _compare(ctx, w2, g2, d_ip2, d_ix2, seed_batch(w2.num_nodes, 64, 9, 0, dtype=np.int64), [15, 10, 5], None, 1.0, 0,
             "after growing")
    ctx.close()


@pytest.mark.parametrize("flags", [a3.A3_TEST_SMALL_GRID, a3.A3_TEST_SMALL_GRID | a3.A3_TEST_FEW_DRAWS])
def test_two_workgroups_per_role_walk_the_node_lists_in_many_rounds(flags):
    """At the benchmark's sizes a wavefront of the sampling kernels serves many nodes in turn, and
    the second launch of a weighted hop reads the marks of its list in several rounds of 64; small
    tests give every node a wavefront of its own.  With the testing flag every role has two
    workgroups: the same loops, many rounds each, in all three kernels and both launch plans."""
    w, g, d_ip, d_ix, seeds = _hub_graph()
    sparse = degree_ranked_cache(g, None, 0.02).cache_map.numpy()
    half = degree_ranked_cache(g, None, 0.5).cache_map.numpy()
    ctx = a3.Context(len(seeds), [15, 3], flags=flags)
    _compare(ctx, w, g, d_ip, d_ix, seeds, [15, 3], None, 1.0, 41, "small grid, uniform")
    _compare(ctx, w, g, d_ip, d_ix, seeds, [15, 3], half, 4.0, 42, "small grid, weighted")
    plans = []
    for b in range(3):     # few neighbours cached: most nodes are left to the second launch, then plan 2
        _compare(ctx, w, g, d_ip, d_ix, seeds, [10, 3], sparse, 8.0, 43 + b, "small grid, sparse cache")
        plans.append(ctx.sample_stats()["launch_plan"])
    assert plans == [1, 2, 2]
    ctx.close()
    w, g, d_ip, d_ix = _graph("mini_copurchase")
    cm = degree_ranked_cache(g, None, 0.2).cache_map.numpy()
    ctx = a3.Context(256, [15, 10, 5], flags=flags)
    for b, gamma in enumerate([1.0, 4.0]):
        _compare(ctx, w, g, d_ip, d_ix, seed_batch(w.num_nodes, 256, 2, b), [15, 10, 5], cm, gamma, b, "small grid")
    ctx.close()


def test_event_brackets_by_kind():
    """A3_PROFILE brackets sampling, retrieve and aggregation; A3_PROFILE_RETRIEVE the retrieve only;
    a plain context none.  One duration per call since the last read, each positive."""
    w, g, d_ip, d_ix = _graph("mini_copurchase")
    full = make_features(g.num_nodes, w.feat_dim, w.feat_dtype, feat_seed=5)
    split = degree_ranked_cache(g, full, 0.2, pin_host=True)
    d_cm, d_fd = split.cache_map.to(DEV), split.feat_dev.to(DEV)
    out = torch.empty((200_000, w.feat_dim), dtype=w.feat_dtype, device=DEV)
    for flags, kinds in [(a3.A3_PROFILE, (0, 1)), (a3.A3_PROFILE_RETRIEVE, (1,)), (0, ())]:
        ctx = a3.Context(w.batch, w.fanouts, flags=flags)
        for b in range(3):
            seeds = torch.from_numpy(seed_batch(w.num_nodes, w.batch, 0, b)).to(DEV)
            ctx.sample_gather_begin(d_ip, d_ix, seeds, w.fanouts, d_cm, 4 * Q, b, d_fd, split.feat_host, out)
            ctx.sample_blocks_end()
        for kind in (0, 1, 2):
            if kind in kinds:
                ms = ctx.profile_read(kind)
                assert len(ms) == 3 and all(0.0 < t < 100.0 for t in ms)
                assert ctx.profile_read(kind) == []
            elif kind == 2 and flags == a3.A3_PROFILE:
                assert ctx.profile_read(kind) == []
            else:
                with pytest.raises(a3.A3Error):
                    ctx.profile_read(kind)
        ctx.close()


def test_one_unit_with_a_bad_seed_retrieves_nothing_and_recovers():
    """A3_VALIDATE finds a repeated seed on the device: the unit's retrieve copies no row, the
    error comes with sample_blocks_end, and the next unit on the context is right again."""
    w, g, d_ip, d_ix = _graph("mini_copurchase")
    full = make_features(g.num_nodes, w.feat_dim, w.feat_dtype, feat_seed=5)
    split = degree_ranked_cache(g, full, 0.2, pin_host=True)
    d_cm, d_fd = split.cache_map.to(DEV), split.feat_dev.to(DEV)
    ctx = a3.Context(64, w.fanouts, flags=a3.A3_VALIDATE)
    out = torch.full((100_000, w.feat_dim), 7.0, dtype=w.feat_dtype, device=DEV)
    bad = torch.tensor([5, 9, 5, 11], dtype=torch.int32, device=DEV)
    ctx.sample_gather_begin(d_ip, d_ix, bad, w.fanouts, d_cm, 4 * Q, 0, d_fd, split.feat_host, out)
    with pytest.raises(a3.A3Error) as ei:
        ctx.sample_blocks_end()
    assert ei.value.code == a3.A3_ERR_INPUT
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
    seeds = seed_batch(w.num_nodes, 64, 3, 1)
    ctx.sample_gather_begin(d_ip, d_ix, torch.from_numpy(seeds).to(DEV), w.fanouts, d_cm, 4 * Q, 1, d_fd,
                            split.feat_host, out)
    got = ctx.sample_blocks_end().to_host()
    torch.cuda.synchronize()
    want = oracle.sample_blocks(g.indptr.numpy(), g.indices.numpy(), seeds, w.fanouts, split.cache_map.numpy(), 4 * Q, 1)
    blocks_equal(got, want)
    want_rows = oracle.gather_features(split.feat_dev.numpy(), split.feat_host.numpy(), split.cache_map.numpy(),
                                       want.input_nodes)
    assert out[: want.n_src[-1]].cpu().numpy().tobytes() == want_rows.tobytes()
    ctx.close()


def test_static_map_contexts_keep_what_they_derived_from_the_map():
    """A3_STATIC_MAP: the bitmap of cached nodes and the weight classes are made when the map's
    pointer changes, not at every call; calls on one map, on another, without weights in between,
    after a FIFO update through the context (which rewrites the map in place), all equal the oracle"""
    w, g, d_ip, d_ix = _graph("mini_copurchase")
    maps = [degree_ranked_cache(g, None, f).cache_map for f in (0.2, 0.6, 1.0)]
    d_maps = [m.to(DEV) for m in maps]
    ctx = a3.Context(128, [15, 10, 5], flags=a3.A3_STATIC_MAP)

    def call(k, b, gamma=4.0, fan=(15, 10, 5)):
        seeds = seed_batch(w.num_nodes, 128 - b, 6, b)
        got = ctx.sample_blocks(d_ip, d_ix, torch.from_numpy(seeds).to(DEV), list(fan), d_maps[k], int(gamma * Q), b)
        want = oracle.sample_blocks(g.indptr.numpy(), g.indices.numpy(), seeds, list(fan), d_maps[k].cpu().numpy(),
                                    int(gamma * Q), b)
        blocks_equal(got.to_host(), want)
        return ctx.sample_stats()["weight_classes"]

    assert [call(0, b) for b in range(3)] == [3, 3, 3]        # made once, kept twice
    assert call(1, 3) == 3 and call(1, 4, fan=(3, 2)) == 3     # another map
    assert call(2, 5) == 1                                      # everything cached: one class
    assert call(0, 6, gamma=1.0) == 0                           # no weights in between
    assert call(0, 7) == 3
    # the map rewritten in place by this context's FIFO update: noticed without a new pointer
    N, n_slots = w.num_nodes, 500
    cm = (-torch.arange(N, dtype=torch.int32) - 1).to(DEV)
    d_maps.append(cm)
    owner = torch.full((n_slots,), -1, dtype=torch.int32, device=DEV)
    state = torch.zeros(4, dtype=torch.int32, device=DEV)
    cache = torch.zeros((n_slots, 4), dtype=torch.float32, device=DEV)
    rows = torch.zeros((N, 4), dtype=torch.float32, device=DEV)
    classes = []
    for b in range(8, 11):
        classes.append(call(3, b))
        ctx.cache_fifo_update(cm, owner, state, cache, rows)
        torch.cuda.synchronize()
    assert classes == [2, 3, 3]                                 # empty cache first, then both classes
    # the caller rewrites a map in place: announced
    d_maps[0].copy_(d_maps[2])
    ctx.device_map_changed()
    assert call(0, 11) == 1
    ctx.close()


def test_isolated_nodes_and_no_eids():
    indptr = torch.tensor([0, 0, 1, 2, 2], dtype=torch.int64)
    indices = torch.tensor([2, 1], dtype=torch.int64)
    ctx = a3.Context(4, [4, 4], flags=a3.A3_NO_EIDS)
    seeds = torch.tensor([0, 1, 3], dtype=torch.int64)
    got = ctx.sample_blocks(indptr.to(DEV), indices.to(DEV), seeds.to(DEV), [4, 4], None, Q, 0)
    assert all(e is None for e in got.blk_eids)
    want = oracle.sample_blocks(indptr.numpy(), indices.numpy(), seeds.numpy(), [4, 4])
    h = got.to_host()
    h.blk_eids = want.blk_eids
    blocks_equal(h, want)
    ctx.close()


def test_repeated_calls_are_byte_identical_and_seed_sensitive():
    w, g, d_ip, d_ix = _graph("mini_copurchase")
    ctx = a3.Context(w.batch, w.fanouts)
    seeds = torch.from_numpy(seed_batch(w.num_nodes, w.batch, 0, 0)).to(DEV)
    a = ctx.sample_blocks(d_ip, d_ix, seeds, w.fanouts, None, Q, 7).to_host()
    b = ctx.sample_blocks(d_ip, d_ix, seeds, w.fanouts, None, Q, 7).to_host()
    blocks_equal(a, b)
    c = ctx.sample_blocks(d_ip, d_ix, seeds, w.fanouts, None, Q, 8).to_host()
    assert not np.array_equal(a.blk_eids[0], c.blk_eids[0])
    ctx.close()


@pytest.mark.parametrize("dim,dtype", [(64, torch.float32), (602, torch.float32), (100, torch.float32),
                                       (128, torch.float16), (3, torch.float16), (1, torch.float16),
                                       (5, torch.float32),
                                       # rows that are 4- or 8-byte aligned and >= 64 bytes: 16-byte
                                       # accesses plus a tail of 1-3 dwords, 1..8 vectors per lane,
                                       # and more than one column step (n16 > 512)
                                       (602, torch.float16), (17, torch.float32), (23, torch.float32),
                                       (34, torch.float16), (2050, torch.float32), (4102, torch.float32),
                                       (1538, torch.float16)])
def test_gather_matches_oracle(dim, dtype):
    w, g, _, _ = _graph("tiny")
    full = make_features(g.num_nodes, dim, dtype, feat_seed=2)
    ctx = a3.Context(16, [2])
    for frac, host_workgroups in [(1.0, 0), (0.2, 0), (0.2, 5), (0.0, 0)]:
        ctx.set_gather_host_workgroups(host_workgroups)   # 5: host rows by workgroups of their own
        split = degree_ranked_cache(g, full, frac, pin_host=True)
        d_cm = split.cache_map.to(DEV)
        d_fd = None if split.feat_dev is None else split.feat_dev.to(DEV)
        for n_ids, idt in [(0, np.int32), (1, np.int64), (777, np.int32), (5000, np.int64)]:
            print(f"[case] gather dim={dim} {dtype} frac={frac} host_workgroups={host_workgroups} "
                  f"n_ids={n_ids} idx={idt.__name__}", flush=True)
            ids = seed_batch(g.num_nodes, n_ids, 4, n_ids, dtype=idt) if n_ids else np.zeros(0, dtype=idt)
            got = ctx.gather_features(d_fd, split.feat_host, d_cm, torch.from_numpy(ids).to(DEV))
            torch.cuda.synchronize()
            fd = None if split.feat_dev is None else split.feat_dev.numpy()
            fh = None if split.feat_host is None else split.feat_host.numpy()
            want = oracle.gather_features(fd, fh, split.cache_map.numpy(), ids)
            assert got.cpu().numpy().tobytes() == want.tobytes()
    # no device map: rows are addressed by id in the device store
    ids = seed_batch(g.num_nodes, 999, 4, 1, dtype=np.int32)
    got = ctx.gather_features(full.to(DEV), None, None, torch.from_numpy(ids).to(DEV))
    want = oracle.gather_features(full.numpy(), None, None, ids)
    assert got.cpu().numpy().tobytes() == want.tobytes()
    ctx.close()


def test_split_call_and_device_count_gather_match_oracle():
    """begin -> gather of the input nodes (count read on the device) -> end"""
    w, g, d_ip, d_ix = _graph("mini_copurchase")
    full = make_features(g.num_nodes, w.feat_dim, w.feat_dtype, feat_seed=5)
    split = degree_ranked_cache(g, full, 0.2, pin_host=True)
    d_cm, d_fd = split.cache_map.to(DEV), split.feat_dev.to(DEV)
    ctx = a3.Context(w.batch, w.fanouts)
    with pytest.raises(a3.A3Error):
        ctx.sample_blocks_end()                      # nothing begun
    with pytest.raises(a3.A3Error):
        ctx.gather_input_features(d_fd, split.feat_host, d_cm,
                                  torch.empty((4, w.feat_dim), dtype=w.feat_dtype, device=DEV))
    for b, cap in [(0, 200_000), (1, 200_000), (2, 1000)]:
        seeds = seed_batch(w.num_nodes, w.batch, 0, b)
        out = torch.full((cap, w.feat_dim), 7.0, dtype=w.feat_dtype, device=DEV)
        ctx.sample_blocks_begin(d_ip, d_ix, torch.from_numpy(seeds).to(DEV), w.fanouts, d_cm, 4 * Q, b)
        with pytest.raises(a3.A3Error):              # a second begin before end is refused
            ctx.sample_blocks_begin(d_ip, d_ix, torch.from_numpy(seeds).to(DEV), w.fanouts, d_cm, 4 * Q, b)
        ctx.gather_input_features(d_fd, split.feat_host, d_cm, out)
        got = ctx.sample_blocks_end().to_host()
        torch.cuda.synchronize()
        want = oracle.sample_blocks(g.indptr.numpy(), g.indices.numpy(), seeds, w.fanouts,
                                    split.cache_map.numpy(), 4 * Q, b)
        blocks_equal(got, want)
        n = min(cap, want.n_src[-1])
        want_rows = oracle.gather_features(split.feat_dev.numpy(), split.feat_host.numpy(),
                                           split.cache_map.numpy(), want.input_nodes[:n])
        assert out[:n].cpu().numpy().tobytes() == want_rows.tobytes()
        assert bool((out[n:] == 7.0).all()), "rows beyond the count or the capacity stay untouched"
    ctx.close()


@pytest.mark.parametrize("name,frac", [("mini_copurchase", 0.2), ("mini_citation", 1.0), ("mini_social", 0.6), ("tiny", 0.0)])
def test_sampling_and_retrieve_as_one_unit_match_oracle(name, frac):
    """a3_sample_gather_begin: the rows of a hop's nodes travel on a second stream while the next
    hop is sampled; blocks and rows equal the oracle's for 1 to 4 hops, both stores, both id widths,
    an output buffer that is too small, an empty batch, and with ordinary calls in between"""
    w, g, d_ip, d_ix = _graph(name)
    idt = g.indices.numpy().dtype
    full = make_features(g.num_nodes, w.feat_dim, w.feat_dtype, feat_seed=5)
    split = degree_ranked_cache(g, full, frac, pin_host=True)
    d_cm = split.cache_map.to(DEV)
    d_fd = None if split.feat_dev is None else split.feat_dev.to(DEV)
    fd_np = None if split.feat_dev is None else split.feat_dev.numpy()
    fh_np = None if split.feat_host is None else split.feat_host.numpy()
    ctx = a3.Context(w.batch, [15, 10, 5, 2])
    cases = [([15, 10, 5], 200_000, w.batch, 4.0), ([10], 200_000, w.batch, 1.0), ([3, 2, 2, 2], 200_000, w.batch // 2, 2.0),
             ([15, 10], 700, w.batch, 4.0), ([15, 10, 5], 200_000, 0, 4.0), ([15, 10, 5], 200_000, w.batch, 8.0)]
    for b, (fan, cap, n_seeds, gamma) in enumerate(cases):
        print(f"[case] one unit graph={name} fanouts={fan} out rows={cap} seeds={n_seeds} gamma={gamma}", flush=True)
        seeds = seed_batch(w.num_nodes, n_seeds, 4, b, dtype=idt)
        out = torch.full((cap, w.feat_dim), 7.0, dtype=w.feat_dtype, device=DEV)
        ctx.sample_gather_begin(d_ip, d_ix, torch.from_numpy(seeds).to(DEV), fan, d_cm, int(gamma * Q), b,
                                d_fd, split.feat_host, out)
        with pytest.raises(a3.A3Error):              # a second begin before end is refused
            ctx.sample_gather_begin(d_ip, d_ix, torch.from_numpy(seeds).to(DEV), fan, d_cm, int(gamma * Q), b,
                                    d_fd, split.feat_host, out)
        got = ctx.sample_blocks_end().to_host()
        torch.cuda.synchronize()
        want = oracle.sample_blocks(g.indptr.numpy(), g.indices.numpy(), seeds, fan, split.cache_map.numpy(),
                                    int(gamma * Q), b)
        blocks_equal(got, want)
        n = min(cap, want.n_src[-1])
        want_rows = oracle.gather_features(fd_np, fh_np, split.cache_map.numpy(), want.input_nodes[:n])
        assert out[:n].cpu().numpy().tobytes() == want_rows.tobytes()
        assert bool((out[n:] == 7.0).all()), "rows beyond the count or the capacity stay untouched"
        if b == 2:   # an ordinary call in between
            _compare(ctx, w, g, d_ip, d_ix, seeds, fan, split.cache_map.numpy(), gamma, b, "between units")
    ctx.close()


@pytest.mark.parametrize("host_workgroups", [0, 16, 3])
@pytest.mark.parametrize("dim,dtype", [(100, torch.float32), (602, torch.float32), (8, torch.float16)])
def test_gather_partly_cached_many_rows_and_missing_stores(dim, dtype, host_workgroups):
    """more rows than the workgroups set aside for host rows see in one round, repeated ids,
    every cache fraction with both stores given; then a store withheld: its rows stay untouched"""
    w, g, _, _ = _graph("tiny")
    full = make_features(g.num_nodes, dim, dtype, feat_seed=9)
    rng = np.random.default_rng(dim)
    ids = rng.integers(0, g.num_nodes, size=70_001).astype(np.int32)
    d_ids = torch.from_numpy(ids).to(DEV)
    ctx = a3.Context(16, [2])
    ctx.set_gather_host_workgroups(host_workgroups)
    with pytest.raises(a3.A3Error):
        ctx.set_gather_host_workgroups(1025)
    spare_host = torch.zeros((1, dim), dtype=dtype).pin_memory()
    spare_dev = torch.zeros((1, dim), dtype=dtype, device=DEV)
    for frac in [1.0, 0.95, 0.3, 0.0]:
        print(f"[case] gather many rows dim={dim} {dtype} frac={frac} host_workgroups={host_workgroups}", flush=True)
        split = degree_ranked_cache(g, full, frac, pin_host=True)
        d_cm = split.cache_map.to(DEV)
        d_fd = spare_dev if split.feat_dev is None else split.feat_dev.to(DEV)
        f_h = spare_host if split.feat_host is None else split.feat_host
        got = ctx.gather_features(d_fd, f_h, d_cm, d_ids)
        torch.cuda.synchronize()
        fd = None if split.feat_dev is None else split.feat_dev.numpy()
        fh = None if split.feat_host is None else split.feat_host.numpy()
        want = oracle.gather_features(fd, fh, split.cache_map.numpy(), ids)
        assert got.cpu().numpy().tobytes() == want.tobytes()
        if 0.0 < frac < 1.0:
            cached = split.cache_map.numpy()[ids] >= 0
            for keep_dev in (True, False):
                out = torch.full((len(ids), dim), 7.0, dtype=dtype, device=DEV)
                ctx.gather_features(d_fd if keep_dev else None, None if keep_dev else f_h, d_cm, d_ids, out=out)
                o = out.cpu().numpy()
                mine = cached if keep_dev else ~cached
                assert o[mine].tobytes() == want[mine].tobytes()
                assert np.all(o[~mine] == 7.0)
    ctx.close()


def test_gather_unaligned_buffers_fall_back_to_narrow_copies():
    w, g, _, _ = _graph("tiny")
    full = make_features(g.num_nodes, 66, torch.float16, feat_seed=3)   # 132-byte rows: 4-byte vectors
    ctx = a3.Context(16, [2])
    ids = seed_batch(g.num_nodes, 1234, 4, 2, dtype=np.int32)
    d_full = full.to(DEV)
    backing = torch.empty(1234 * 66 + 1, dtype=torch.float16, device=DEV)
    out = backing[1:].view(1234, 66)                                  # 2-byte aligned output
    got = ctx.gather_features(d_full, None, None, torch.from_numpy(ids).to(DEV), out=out)
    want = oracle.gather_features(full.numpy(), None, None, ids)
    assert got.cpu().numpy().tobytes() == want.tobytes()
    ctx.close()
