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
from workloads import get_config, make_graph, make_features, degree_ranked_cache, seed_batch

pytestmark = pytest.mark.gpu
Q = 65536
DEV = "cuda:0"


def _run(name, gammas, check_rows, n_batches=1):
    w = get_config(name)
    t0 = time.time()
    g = make_graph(w.num_nodes, w.mean_degree, w.d_min, w.d_max, w.a, w.symmetric, w.graph_seed,
                   w.idx_dtype, device=DEV)
    full = make_features(w.num_nodes, w.feat_dim, w.feat_dtype, device=DEV)
    split = degree_ranked_cache(g, full, w.cache_frac, pin_host=True)
    torch.cuda.synchronize()
    print(f"[gen] {name}: {g.stats()} cached={split.n_cached} in {time.time() - t0:.1f}s", flush=True)
    ip_h, ix_h = g.indptr.cpu().numpy(), g.indices.cpu().numpy()
    cm_h = split.cache_map.cpu().numpy()
    idt = ix_h.dtype
    ctx = a3.Context(w.batch, w.fanouts)
    for gamma in gammas:
        for b in range(n_batches):
            seeds = seed_batch(w.num_nodes, w.batch, 0, b, dtype=idt)
            print(f"[case] {name} gamma={gamma} batch={b}", flush=True)
            t0 = time.time()
            got_d = ctx.sample_blocks(g.indptr, g.indices, torch.from_numpy(seeds).to(DEV), w.fanouts,
                                      split.cache_map, int(gamma * Q), b)
            rows = ctx.gather_features(split.feat_dev, split.feat_host, split.cache_map,
                                       got_d.input_nodes)
            torch.cuda.synchronize()
            t1 = time.time()
            got = got_d.to_host()
            want = oracle.sample_blocks(ip_h, ix_h, seeds, w.fanouts, cm_h, int(gamma * Q), b)
            t2 = time.time()
            print(f"[time] gpu {t1 - t0:.3f}s oracle {t2 - t1:.1f}s edges={want.n_edges} "
                  f"n_src={want.n_src}", flush=True)
            blocks_equal(got, want)
            if b == 0 and gamma == gammas[0]:
                check_block_invariants(ip_h, ix_h, seeds, w.fanouts, got)
            # gathered rows: every row against the generator's table through the split, via the oracle
            ids = want.input_nodes
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
    ctx.close()


def test_social_full_size():
    _run("social", [1.0], check_rows=1 << 30)


def test_copurchase_full_size_uniform_and_biased():
    _run("copurchase", [1.0, 4.0], check_rows=1 << 30)


def test_citation_full_size():
    _run("citation", [1.0], check_rows=200_000)
