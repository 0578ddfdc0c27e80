"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times:
graphs are generated on the GPU, mini-batches go through the HIP library and through the CPU
oracle, and every output array is compared (bit-exact / byte-exact).  Covers the dense social
graph, the co-purchase graph with its batch x cache x bias-rate sweep at the corner cells, the
citation-scale graph with 8-byte ids (all three hops against the full oracle), one full-size
mini-batch through a stream pipeline and the block mean, the cache policies on the co-purchase
graph, and the multi-threaded host sampler in the vector form the GPU machine's CPU picks."""
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2511_07421_amd as a3
from helpers import blocks_equal, check_block_invariants
from workloads import (get_config, make_graph, make_features, degree_ranked_cache, padded_rows,
                       seed_batch)

pytestmark = pytest.mark.gpu
Q = 65536
DEV = "cuda:0"
_worlds = {}


class World:
    """one workload generated on the GPU, with host copies of what the oracle reads"""

    def __init__(self, name, say):
        w = get_config(name)
        t0 = time.time()
        self.w = w
        self.g = make_graph(w.num_nodes, w.mean_degree, w.d_min, w.d_max, w.a, w.symmetric, w.graph_seed,
                            w.idx_dtype, device=DEV)
        self.full = make_features(w.num_nodes, w.feat_dim, w.feat_dtype, device=DEV)
        torch.cuda.synchronize()
        self.ip_h, self.ix_h = self.g.indptr.cpu().numpy(), self.g.indices.cpu().numpy()
        self.splits = {}
        say(f"[gen] {name}: {self.g.stats()} in {time.time() - t0:.1f}s")

    def split(self, frac):
        """the degree-ranked cache at this fraction, rows padded to 128 bytes as bench.py does"""
        if frac not in self.splits:
            self.splits.clear()        # one split at a time: the host store is pinned memory
            s = degree_ranked_cache(self.g, self.full, frac, pin_host=True, row_align=128)
            self.splits[frac] = (s, s.cache_map.cpu().numpy())
        return self.splits[frac]


def _world(name, say):
    if name not in _worlds:
        _worlds.clear()                # one full-size workload on the GPU at a time
        torch.cuda.empty_cache()
        _worlds[name] = World(name, say)
    return _worlds[name]


def _cap_rows(w, batch):
    cap = batch
    for f in w.fanouts:
        cap *= 1 + f
    return min(cap, w.num_nodes)


def _check_rows(world, split, cm_h, ids, rows, check_rows):
    """gathered rows against the oracle's copy; the oracle reads host arrays, so it is handed
    only the rows it will touch, renumbered"""
    if check_rows < ids.shape[0]:
        pick = np.unique(np.linspace(0, ids.shape[0] - 1, check_rows).astype(np.int64))
    else:
        pick = np.arange(ids.shape[0])
    c = cm_h[ids[pick]]
    dev_rows = np.unique(c[c >= 0])
    host_rows = np.unique(-c[c < 0] - 1)
    fd_small = split.feat_dev[torch.from_numpy(dev_rows).to(DEV)].cpu().numpy() if dev_rows.size else None
    fh_small = split.feat_host[torch.from_numpy(host_rows)].numpy() if host_rows.size else None
    cm_small = np.zeros_like(c)
    cm_small[c >= 0] = np.searchsorted(dev_rows, c[c >= 0])
    cm_small[c < 0] = -np.searchsorted(host_rows, -c[c < 0] - 1) - 1
    want_rows = oracle.gather_features(fd_small, fh_small, cm_small, np.arange(pick.shape[0], dtype=np.int64))
    got_rows = rows[torch.from_numpy(pick).to(DEV)].cpu().numpy()
    assert got_rows.tobytes() == want_rows.tobytes()


def _run(say, name, cells, check_rows, validate=False, host_sampler=False):
    """cells: (batch, cache fraction, bias rate, mini-batch number) compared one by one"""
    world = _world(name, say)
    w, g = world.w, world.g
    idt = world.ix_h.dtype
    max_batch = max(c[0] for c in cells)
    ctx = a3.Context(max_batch, w.fanouts)
    out = padded_rows(_cap_rows(w, max_batch), w.feat_dim, w.feat_dtype, DEV, 128)
    if validate:      # the generators' outputs satisfy what the sampler takes on trust, at full size
        ctx.validate_graph(g.indptr, g.indices)
    for batch, frac, gamma, b in cells:
        split, cm_h = world.split(frac)
        if validate:
            ctx.validate_cache_map(split.cache_map, split.n_cached, w.num_nodes - split.n_cached)
        seeds = seed_batch(w.num_nodes, batch, 0, b, dtype=idt)
        t0 = time.time()
        # the step exactly as bench.py queues it: sampling and the retrieve of its input rows as one
        # unit (row counts taken on the device; where rows sit in host memory, those of earlier
        # hops on a second stream beside the sampling of later hops), then the wait for the counts
        ctx.sample_gather_begin(g.indptr, g.indices, torch.from_numpy(seeds).to(DEV), w.fanouts,
                                split.cache_map, int(gamma * Q), b, split.feat_dev, split.feat_host, out)
        got_d = ctx.sample_blocks_end()
        rows = out[: got_d.n_src[-1]]
        torch.cuda.synchronize()
        t1 = time.time()
        got = got_d.to_host()
        say(f"[case] {name} batch={batch} cache={frac} gamma={gamma} mini-batch={b}: gpu {t1 - t0:.3f}s, "
            f"edges={got.n_edges} n_src={got.n_src}; oracle running")
        want = oracle.sample_blocks(world.ip_h, world.ix_h, seeds, w.fanouts, cm_h, int(gamma * Q), b)
        say(f"[time] oracle {time.time() - t1:.1f}s")
        blocks_equal(got, want)
        if (batch, frac, gamma, b) == cells[0]:
            check_block_invariants(world.ip_h, world.ix_h, seeds, w.fanouts, got)
        _check_rows(world, split, cm_h, want.input_nodes, rows, check_rows)
        if split.feat_host is not None and (batch, frac, gamma, b) == cells[0]:
            # the same retrieve with workgroups set aside for the host rows (as the pipelines'
            # workers run it) and every id looked up in the map: the same rows, all of them
            ctx.set_gather_host_workgroups(16)
            again = torch.zeros((got_d.n_src[-1], w.feat_dim), dtype=w.feat_dtype, device=DEV)
            ctx.gather_features(split.feat_dev, split.feat_host, split.cache_map, got_d.input_nodes, out=again)
            ctx.set_gather_host_workgroups(0)
            assert torch.equal(again, rows)
            del again
        if host_sampler:
            # the host sampler as bench.py's cpu_sampler leg runs it (16 threads, the vector form
            # this machine's CPU picks): the same blocks
            cpu = a3.CpuSampler(16)
            blocks_equal(cpu.sample_blocks(world.ip_h, world.ix_h, seeds, w.fanouts, cm_h, int(gamma * Q), b), want)
            cpu.close()
            say("[case] host sampler, 16 threads: equal")
    ctx.close()


def test_social_full_size(progress):
    _run(progress, "social", [(1024, 1.0, 1.0, 0)], check_rows=1 << 30, validate=True, host_sampler=True)


def test_social_full_size_pipeline_and_block_mean(progress):
    """one full-size mini-batch through a3_pipeline_* (mode 1, two workers, the second worker busy
    with another mini-batch) and a3_block_mean_of_hop, element by element against the oracle"""
    world = _world("social", progress)
    w, g = world.w, world.g
    split, cm_h = world.split(1.0)
    cap = _cap_rows(w, w.batch)
    outs = [padded_rows(cap, w.feat_dim, w.feat_dtype, DEV, 128) for _ in range(2)]
    pipe = a3.Pipeline(a3.A3_PIPE_MODE1, 2, w.batch, w.fanouts)
    seeds = [seed_batch(w.num_nodes, w.batch, 0, b, dtype=np.int32) for b in (3, 4)]
    torch.cuda.synchronize()
    for k in range(2):
        pipe.submit(g.indptr, g.indices, torch.from_numpy(seeds[k]).to(DEV), w.fanouts, split.cache_map, Q, 3 + k,
                    split.feat_dev, split.feat_host, outs[k])
    blk = pipe.wait()
    got = blk.to_host()
    progress(f"[case] social mini-batch 3 through pipeline mode 1: edges={got.n_edges}; oracle running")
    want = oracle.sample_blocks(world.ip_h, world.ix_h, seeds[0], w.fanouts, cm_h, Q, 3)
    blocks_equal(got, want)
    rows = outs[0][: got.n_src[-1]]
    _check_rows(world, split, cm_h, want.input_nodes, rows, 1 << 30)
    pipe.wait()
    pipe.close()
    # the block mean of the outermost hop, queued as bench.py queues it (counts on the device)
    ctx = a3.Context(w.batch, w.fanouts)
    H = len(w.fanouts)
    agg = padded_rows(want.n_dst[-1], w.feat_dim, w.feat_dtype, DEV, 128)
    ctx.sample_blocks_begin(g.indptr, g.indices, torch.from_numpy(seeds[0]).to(DEV), w.fanouts, split.cache_map, Q, 3)
    ctx.gather_input_features(split.feat_dev, split.feat_host, split.cache_map, outs[1])
    ctx.block_mean_of_hop(H - 1, outs[1], agg)
    blocks_equal(ctx.sample_blocks_end().to_host(), want)
    torch.cuda.synchronize()
    x = world.full[torch.from_numpy(want.input_nodes).to(DEV)].cpu().numpy()
    m_want = oracle.block_mean(want.blk_indptr[-1], want.blk_indices[-1], x)
    S = oracle.block_mean(want.blk_indptr[-1], want.blk_indices[-1], np.abs(x))
    deg = np.diff(want.blk_indptr[-1]).astype(np.float64)[:, None]
    # d fp32 additions in edge order and one division: (d + 1) roundings of 2^-24 on sums bounded
    # by sum |x| = d * mean |x|
    tol = (deg + 1) * 2.0 ** -24 * S * 1.0000001
    m_got = agg.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(m_got - m_want) <= tol)
    progress("[case] social block mean of the outermost hop: within the bound")
    ctx.close()


def test_copurchase_full_size_uniform_and_biased(progress):
    _run(progress, "copurchase", [(4096, 0.2, 1.0, 0), (4096, 0.2, 4.0, 0)], check_rows=1 << 30, validate=True)


@pytest.mark.parametrize("batch,frac,gamma", [(16384, 0.05, 8.0), (256, 0.5, 2.0), (1024, 1.0, 4.0)])
def test_copurchase_sweep_corner_cells(progress, batch, frac, gamma):
    """corner cells of the batch x cache x bias-rate sweep: the largest batch (launch bounds above
    one million frontier nodes and 1 024 scan tiles, so the tile sums go through k_scan_tiles
    instead of being scanned by their consumers) with the smallest cache and the largest bias rate,
    the smallest batch, and a full cache (one weight class: the bias rate must not matter)"""
    _run(progress, "copurchase", [(batch, frac, gamma, 1)], check_rows=300_000)


def test_copurchase_full_size_fifo_cache_and_access_counts(progress):
    """Cache policies at full size: a FIFO ring of 2.5 % of the nodes that starts empty (every
    mini-batch brings more misses than it has slots) and three mini-batches of locality-aware
    sampling that read it: the first meets one weight class, the second finds few neighbours
    cached and leaves half of its wide nodes to the second sampling launch, so the third runs the
    single full launch per hop.  The update goes through both entry points; the access counts of
    the same mini-batches and the ranked fill are compared too.  Blocks, rows, map, owners, ring
    head and counts equal the oracle's after every step."""
    world = _world("copurchase", progress)
    w, g = world.w, world.g
    N, batch = w.num_nodes, 1024
    n_slots = N // 40
    full_h = world.full.cpu()
    host_all = full_h.pin_memory()
    full_np = full_h.numpy()
    ctx = a3.Context(batch, w.fanouts)
    cm = -torch.arange(N, dtype=torch.int32, device=DEV) - 1
    owner = torch.full((n_slots,), -1, dtype=torch.int32, device=DEV)
    state = torch.zeros(4, dtype=torch.int32, device=DEV)
    cache = torch.zeros((n_slots, w.feat_dim), dtype=w.feat_dtype, device=DEV)
    rows = torch.zeros((_cap_rows(w, batch), w.feat_dim), dtype=w.feat_dtype, device=DEV)
    counts = torch.zeros(N, dtype=torch.int32, device=DEV)
    o_cm = (-np.arange(N) - 1).astype(np.int32)
    o_owner = np.full(n_slots, -1, dtype=np.int32)
    o_head = np.zeros(1, dtype=np.int32)
    o_cache = np.zeros((n_slots, w.feat_dim), dtype=np.float32)
    o_counts = np.zeros(N, dtype=np.uint32)
    plans = []
    for b in range(3):
        seeds = seed_batch(N, batch, 0, 40 + b, dtype=np.int32)
        ctx.sample_blocks_begin(g.indptr, g.indices, torch.from_numpy(seeds).to(DEV), w.fanouts, cm, 4 * Q, b)
        ctx.gather_input_features(cache, host_all, cm, rows)
        ctx.cache_count_accesses(counts)
        ctx.cache_fifo_update(cm, owner, state, cache, rows, static_scratch=(b == 1))
        blk = ctx.sample_blocks_end()
        st = ctx.sample_stats()
        plans.append((st["launch_plan"], st["deferred_wide_nodes"] + st["deferred_hubs"]))
        progress(f"[case] copurchase fifo step {b}: edges={blk.n_edges} n_src={blk.n_src} stats={st}; oracle running")
        ob = oracle.sample_blocks(world.ip_h, world.ix_h, seeds, w.fanouts, o_cm, 4 * Q, b)
        blocks_equal(blk.to_host(), ob)
        ids = ob.input_nodes.astype(np.int32)
        # the oracle reads host arrays: hand it the rows it will touch, renumbered (the cache's rows
        # first, then the host store's)
        c = o_cm[ids]
        dev_rows, host_rows = np.unique(c[c >= 0]), np.unique(-c[c < 0] - 1)
        cm_small = np.where(c >= 0, np.searchsorted(dev_rows, np.maximum(c, 0)),
                            -np.searchsorted(host_rows, np.maximum(-c - 1, 0)) - 1).astype(np.int32)
        o_rows = oracle.gather_features(o_cache[dev_rows] if dev_rows.size else None,
                                        full_np[host_rows] if host_rows.size else None, cm_small,
                                        np.arange(ids.shape[0], dtype=np.int64))
        oracle.count_accesses(ids, o_counts)
        misses = oracle.cache_fifo_update(o_cm, o_owner, o_head, o_cache, ids, o_rows)
        torch.cuda.synchronize()
        assert rows[: blk.n_src[-1]].cpu().numpy().tobytes() == o_rows.tobytes()
        sv = state.cpu().numpy()
        assert sv[0] == o_head[0] and sv[1] == misses
        assert np.array_equal(cm.cpu().numpy(), o_cm)
        assert np.array_equal(owner.cpu().numpy(), o_owner)
        filled = o_owner >= 0
        assert np.array_equal(cache.cpu().numpy()[filled], o_cache[filled])
    assert plans[0] == (1, 0) and plans[1][0] == 1 and plans[1][1] > 10_000 and plans[2] == (2, 0)
    assert np.array_equal(counts.cpu().numpy().view(np.uint32), o_counts)
    got_cm, got_order = ctx.cache_rank(counts, n_slots)
    want_cm, want_order = oracle.rank_cache(o_counts, n_slots)
    assert np.array_equal(got_cm.cpu().numpy(), want_cm)
    assert np.array_equal(got_order.cpu().numpy(), want_order)
    ctx.close()


def test_citation_full_size(progress):
    _run(progress, "citation", [(8192, 1.0, 1.0, 0)], check_rows=200_000, validate=True)
