"""Seeded random configurations against the oracle: graphs of several sizes, degree ranges and
id widths, 1-3 hops, fanouts 1-64, every cache fraction (degree-ranked and arbitrary cached sets),
bias rates from 1 to 1000; tables of several widths and types through the retrieve with and
without workgroups set aside for host rows, and through sampling and retrieve as one unit.  Equality throughout; what the fixed cases of the other
files do not happen to combine, these do."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_07421_amd as a3
from helpers import blocks_equal
from workloads import make_graph, degree_ranked_cache, seed_batch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_sampling_configurations(seed):
    rng = np.random.default_rng(seed)
    for _ in range(4):
        N = int(rng.choice([300, 2000, 12000, 40000]))
        mean = min(float(rng.choice([3.0, 12.0, 60.0, 300.0, 900.0])), N / 4)
        dmax = int(min(N - 1, rng.choice([50, 500, 6000, 20000])))
        idt = torch.int32 if rng.integers(0, 2) else torch.int64
        g = make_graph(N, mean, 1, max(dmax, 2), 2.1, bool(rng.integers(0, 2)), int(rng.integers(0, 1 << 30)), idt)
        ip, ix = g.indptr.numpy(), g.indices.numpy()
        d_ip, d_ix = g.indptr.to(DEV), g.indices.to(DEV)
        for rep in range(5):
            fan = [int(rng.choice([1, 2, 3, 5, 10, 15, 25, 40, 64])) for _ in range(int(rng.integers(1, 4)))]
            n_seeds = min(int(rng.choice([1, 7, 64, 300])), N)
            frac = float(rng.choice([0.0, 0.03, 0.2, 0.5, 0.9, 1.0]))
            gamma = float(rng.choice([1.0, 1.25, 2.0, 4.0, 8.0, 33.0, 1000.0]))
            rs = int(rng.integers(0, 1 << 40))
            cm = degree_ranked_cache(g, None, frac).cache_map
            if rng.integers(0, 4) == 0:   # an arbitrary cached set instead of the hubs
                cm = cm[torch.from_numpy(rng.permutation(N)).long()].contiguous()
            seeds = seed_batch(N, n_seeds, int(rng.integers(0, 100)), rep, dtype=ix.dtype)
            print(f"[case] random sampling seed={seed} N={N} mean={mean} dmax={dmax} {idt} fan={fan} "
                  f"seeds={n_seeds} frac={frac} gamma={gamma} rs={rs}", flush=True)
            ctx = a3.Context(n_seeds, fan)
            got = ctx.sample_blocks(d_ip, d_ix, torch.from_numpy(seeds).to(DEV), fan, cm.to(DEV),
                                    int(gamma * 65536), rs).to_host()
            blocks_equal(got, oracle.sample_blocks(ip, ix, seeds, fan, cm.numpy(), int(gamma * 65536), rs))
            ctx.close()


@pytest.mark.parametrize("seed", [31, 32, 33])
def test_random_units_of_sampling_and_retrieve(seed):
    """a3_sample_gather_begin on random graphs, tables of several widths and types, every cache
    fraction (rows ahead on the second stream whenever a host store exists), 1-3 hops, output
    buffers that are sometimes too small: blocks and rows equal the oracle's"""
    rng = np.random.default_rng(seed)
    for _ in range(4):
        N = int(rng.choice([300, 2000, 12000]))
        mean = min(float(rng.choice([3.0, 12.0, 60.0, 300.0])), N / 4)
        dmax = int(min(N - 1, rng.choice([50, 500, 6000])))
        idt = torch.int32 if rng.integers(0, 2) else torch.int64
        g = make_graph(N, mean, 1, max(dmax, 2), 2.1, bool(rng.integers(0, 2)), int(rng.integers(0, 1 << 30)), idt)
        ip, ix = g.indptr.numpy(), g.indices.numpy()
        d_ip, d_ix = g.indptr.to(DEV), g.indices.to(DEV)
        for rep in range(4):
            dim = int(rng.choice([1, 2, 3, 8, 25, 64, 100, 128, 301, 602]))
            dt = torch.float32 if rng.integers(0, 2) else torch.float16
            full = torch.from_numpy(rng.standard_normal((N, dim)).astype(np.float32)).to(dt)
            frac = float(rng.choice([0.0, 0.1, 0.5, 0.97, 1.0]))
            split = degree_ranked_cache(g, full, frac, pin_host=True)
            fan = [int(rng.choice([1, 2, 5, 10, 15, 25])) for _ in range(int(rng.integers(1, 4)))]
            n_seeds = min(int(rng.choice([1, 7, 64, 300])), N)
            gamma = float(rng.choice([1.0, 2.0, 4.0, 33.0]))
            rs = int(rng.integers(0, 1 << 40))
            cap = int(rng.choice([N, N, max(1, N // 7)]))
            seeds = seed_batch(N, n_seeds, int(rng.integers(0, 100)), rep, dtype=ix.dtype)
            print(f"[case] random unit seed={seed} N={N} {idt} dim={dim} {dt} frac={frac} fan={fan} seeds={n_seeds} "
                  f"gamma={gamma} out rows={cap}", flush=True)
            fd = split.feat_dev.to(DEV) if split.feat_dev is not None and split.feat_dev.shape[0] else None
            fh = split.feat_host if split.feat_host is not None and split.feat_host.shape[0] else None
            out = torch.full((cap, dim), 3.0, dtype=dt, device=DEV)
            ctx = a3.Context(n_seeds, fan)
            ctx.sample_gather_begin(d_ip, d_ix, torch.from_numpy(seeds).to(DEV), fan, split.cache_map.to(DEV),
                                    int(gamma * 65536), rs, fd, fh, out)
            got = ctx.sample_blocks_end().to_host()
            torch.cuda.synchronize()
            want = oracle.sample_blocks(ip, ix, seeds, fan, split.cache_map.numpy(), int(gamma * 65536), rs)
            blocks_equal(got, want)
            n = min(cap, want.n_src[-1])
            want_rows = oracle.gather_features(None if fd is None else split.feat_dev.numpy(),
                                               None if fh is None else split.feat_host.numpy(),
                                               split.cache_map.numpy(), want.input_nodes[:n])
            assert out[:n].cpu().numpy().tobytes() == want_rows.tobytes()
            assert bool((out[n:] == 3.0).all())
            ctx.close()


@pytest.mark.parametrize("seed", [21, 22])
def test_random_retrieve_configurations(seed):
    rng = np.random.default_rng(seed)
    ctx = a3.Context(8, [2])
    for _ in range(40):
        N = int(rng.choice([50, 3000, 60000]))
        dim = int(rng.choice([1, 2, 3, 8, 25, 64, 100, 128, 301, 602, 1030]))
        dt = torch.float32 if rng.integers(0, 2) else torch.float16
        full = torch.from_numpy(rng.standard_normal((N, dim)).astype(np.float32)).to(dt)
        frac = float(rng.choice([0.0, 0.1, 0.5, 0.97, 1.0]))
        perm = rng.permutation(N)
        n_c = int(round(frac * N))
        cm = np.empty(N, dtype=np.int32)
        cm[perm[:n_c]] = np.arange(n_c, dtype=np.int32)
        cm[perm[n_c:]] = -np.arange(N - n_c, dtype=np.int32) - 1
        fd = full[torch.from_numpy(perm[:n_c])].contiguous() if n_c else None
        fh = full[torch.from_numpy(perm[n_c:])].contiguous().pin_memory() if n_c < N else None
        n_ids = int(rng.choice([0, 1, 63, 1000, 30000, 90000]))
        idt = np.int32 if rng.integers(0, 2) else np.int64
        ids = rng.integers(0, N, size=n_ids).astype(idt)
        hw = int(rng.choice([0, 0, 1, 16, 40]))
        ctx.set_gather_host_workgroups(hw)
        print(f"[case] random retrieve seed={seed} N={N} dim={dim} {dt} frac={frac} n_ids={n_ids} "
              f"idx={idt.__name__} host_workgroups={hw}", flush=True)
        got = ctx.gather_features(None if fd is None else fd.to(DEV), fh, torch.from_numpy(cm).to(DEV),
                                  torch.from_numpy(ids).to(DEV))
        torch.cuda.synchronize()
        want = oracle.gather_features(None if fd is None else fd.numpy(), None if fh is None else fh.numpy(), cm, ids)
        assert got.cpu().numpy().tobytes() == want.tobytes()
    ctx.close()
