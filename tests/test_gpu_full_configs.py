"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times:
graphs are generated on the GPU, one mini-batch goes through the HIP library and through the
CPU oracle, and every output array is compared (bit-exact / byte-exact)."""
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


def _compare_last_hop_by_samples(got, want_prefix, ip_h, ix_h, cm_h, fanouts, bias_q16, rng_seed, n_pick):
    """The oracle ran all hops but the last.  The last hop's destinations are its sources
    (identical by the prefix comparison), so any destination's choice can be recomputed alone:
    check n_pick of them one by one with the oracle's per-node selection, and the whole block
    through the invariants (which re-derive the relabelling from the CSR with numpy)."""
    H = len(fanouts)
    h = H - 1
    D = want_prefix.input_nodes                      # destinations of the last hop
    assert got.n_dst[h] == D.shape[0]
    assert np.array_equal(got.input_nodes[:D.shape[0]].astype(np.int64), D)
    rnd = np.random.RandomState(123)
    picks = rnd.choice(D.shape[0], size=min(n_pick, D.shape[0]), replace=False)
    deg_all = ip_h[D + 1] - ip_h[D]
    hubs = np.argsort(deg_all)[-50:]                 # always include the widest rows
    bp, be = got.blk_indptr[h].astype(np.int64), got.blk_eids[h]
    for i in np.concatenate([picks, hubs]):
        v = int(D[i])
        row, deg = int(ip_h[v]), int(ip_h[v + 1] - ip_h[v])
        weights = None
        if cm_h is not None and bias_q16 > 65536 and deg > fanouts[h]:
            nb = ix_h[row:row + deg]
            weights = np.where(cm_h[nb] >= 0, bias_q16, 65536).astype(np.uint32)
        chosen = oracle.select(rng_seed, h, v, deg, fanouts[h], weights)
        assert list(be[bp[i]:bp[i + 1]] - row) == chosen, (i, v, deg)


def _run(name, gammas, check_rows, n_batches=1, full_hops=None):
    w = get_config(name)
    t0 = time.time()
    g = make_graph(w.num_nodes, w.mean_degree, w.d_min, w.d_max, w.a, w.symmetric, w.graph_seed,
                   w.idx_dtype, device=DEV)
    full = make_features(w.num_nodes, w.feat_dim, w.feat_dtype, device=DEV)
    # as bench.py: rows of the stores and of the output padded to a multiple of 128 bytes
    split = degree_ranked_cache(g, full, w.cache_frac, pin_host=True, row_align=128)
    torch.cuda.synchronize()
    print(f"[gen] {name}: {g.stats()} cached={split.n_cached} in {time.time() - t0:.1f}s", flush=True)
    ip_h, ix_h = g.indptr.cpu().numpy(), g.indices.cpu().numpy()
    cm_h = split.cache_map.cpu().numpy()
    idt = ix_h.dtype
    ctx = a3.Context(w.batch, w.fanouts)
    # the generators' outputs satisfy what the sampler takes on trust, at full size
    ctx.validate_graph(g.indptr, g.indices)
    ctx.validate_cache_map(split.cache_map, split.n_cached, w.num_nodes - split.n_cached)
    cap_rows = w.batch
    for f in w.fanouts:
        cap_rows *= 1 + f
    cap_rows = min(cap_rows, w.num_nodes)
    out = padded_rows(cap_rows, w.feat_dim, w.feat_dtype, DEV, 128)
    for gamma in gammas:
        for b in range(n_batches):
            seeds = seed_batch(w.num_nodes, w.batch, 0, b, dtype=idt)
            print(f"[case] {name} gamma={gamma} batch={b}", flush=True)
            t0 = time.time()
            # the step exactly as bench.py queues it: sampling, the gather of its input nodes with
            # the row count taken on the device, then the wait for the counts
            ctx.sample_blocks_begin(g.indptr, g.indices, torch.from_numpy(seeds).to(DEV), w.fanouts,
                                    split.cache_map, int(gamma * Q), b)
            ctx.gather_input_features(split.feat_dev, split.feat_host, split.cache_map, out)
            got_d = ctx.sample_blocks_end()
            rows = out[: got_d.n_src[-1]]
            torch.cuda.synchronize()
            t1 = time.time()
            got = got_d.to_host()
            H = len(w.fanouts)
            if full_hops is None or full_hops >= H:
                want = oracle.sample_blocks(ip_h, ix_h, seeds, w.fanouts, cm_h, int(gamma * Q), b)
                t2 = time.time()
                print(f"[time] gpu {t1 - t0:.3f}s oracle {t2 - t1:.1f}s edges={want.n_edges} "
                      f"n_src={want.n_src}", flush=True)
                blocks_equal(got, want)
                if b == 0 and gamma == gammas[0]:
                    check_block_invariants(ip_h, ix_h, seeds, w.fanouts, got)
                ids = want.input_nodes
            else:
                # the oracle in full on the first hops, by sampled destinations on the rest
                assert full_hops == H - 1
                want = oracle.sample_blocks(ip_h, ix_h, seeds, w.fanouts[:full_hops], cm_h,
                                            int(gamma * Q), b)
                for h in range(full_hops):
                    assert np.array_equal(got.blk_indptr[h], want.blk_indptr[h])
                    assert np.array_equal(got.blk_indices[h], want.blk_indices[h])
                    assert np.array_equal(got.blk_eids[h], want.blk_eids[h])
                assert got.n_src[:full_hops] == want.n_src
                _compare_last_hop_by_samples(got, want, ip_h, ix_h, cm_h, w.fanouts, int(gamma * Q),
                                             b, 4000)
                check_block_invariants(ip_h, ix_h, seeds, w.fanouts, got)
                t2 = time.time()
                print(f"[time] gpu {t1 - t0:.3f}s oracle+checks {t2 - t1:.1f}s edges={got.n_edges} "
                      f"n_src={got.n_src}", flush=True)
                # the oracle did not produce this hop's input nodes, so nothing of them goes to it:
                # sampled rows are compared with the generator's table by plain indexing
                gi = torch.from_numpy(np.unique(np.linspace(0, got.n_src[-1] - 1, check_rows).astype(np.int64))).to(DEV)
                ids_d = got_d.input_nodes.long()[gi]
                assert torch.equal(rows[gi], full[ids_d])
                continue
            # gathered rows: every row against the generator's table through the split, via the oracle
            if check_rows < ids.shape[0]:
                pick = np.unique(np.linspace(0, ids.shape[0] - 1, check_rows).astype(np.int64))
            else:
                pick = np.arange(ids.shape[0])
            fd_rows = None
            sub_ids = ids[pick]
            c = cm_h[sub_ids]
            # the oracle copies from host arrays; hand it only the rows it will touch
            dev_rows = np.unique(c[c >= 0])
            host_rows = np.unique(-c[c < 0] - 1)
            fd_small = split.feat_dev[torch.from_numpy(dev_rows).to(DEV)].cpu().numpy() if dev_rows.size else None
            fh_small = split.feat_host[torch.from_numpy(host_rows)].numpy() if host_rows.size else None
            cm_small = np.zeros_like(c)
            cm_small[c >= 0] = np.searchsorted(dev_rows, c[c >= 0])
            cm_small[c < 0] = -np.searchsorted(host_rows, -c[c < 0] - 1) - 1
            want_rows = oracle.gather_features(fd_small, fh_small, cm_small,
                                               np.arange(pick.shape[0], dtype=np.int64))
            got_rows = rows[torch.from_numpy(pick).to(DEV)].cpu().numpy()
            assert got_rows.tobytes() == want_rows.tobytes()
            if split.feat_host is not None and b == 0:
                # the same retrieve with workgroups set aside for the host rows (as the pipelines'
                # workers run it), at full size: the same rows, all of them
                ctx.set_gather_host_workgroups(16)
                again = torch.zeros((got_d.n_src[-1], w.feat_dim), dtype=w.feat_dtype, device=DEV)
                ctx.gather_features(split.feat_dev, split.feat_host, split.cache_map, got_d.input_nodes, out=again)
                ctx.set_gather_host_workgroups(0)
                assert torch.equal(again, rows)
                del again
    ctx.close()


def test_social_full_size():
    _run("social", [1.0], check_rows=1 << 30)


def test_copurchase_full_size_uniform_and_biased():
    _run("copurchase", [1.0, 4.0], check_rows=1 << 30)


def test_citation_full_size():
    _run("citation", [1.0], check_rows=200_000, full_hops=2)
