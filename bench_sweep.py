#!/usr/bin/env python3
"""Batch / cache / bias-rate sweep on the co-purchase-style graph (one MI355X).

Shows where locality-aware sampling pays off (paper Sec. II-B Motivation 2, Sec. IV-C ablation):
for every batch size x HBM cache fraction x bias rate gamma it reports the cache hit rate of the
input nodes, the number of input rows, the device time of sampling and of the feature gather
(HBM rows + pinned-host rows over PCIe), and the wall time per mini-batch with two mini-batches
in flight (a3_pipeline_*, parallel mode 2: sampling beside the previous retrieve).  Prints a markdown table; the graph is generated once.

    python bench_sweep.py [--steps 10] [--batches 256,1024,4096,16384] [--cache 0.05,0.2,0.5,1.0]
                          [--gammas 1,2,4,8] [--workload copurchase]
"""
import argparse
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    p = argparse.ArgumentParser()
    p.add_argument("--workload", default="copurchase")
    p.add_argument("--steps", type=int, default=10)
    p.add_argument("--warmup", type=int, default=2)
    p.add_argument("--batches", default="256,1024,4096,16384")
    p.add_argument("--cache", default="0.05,0.2,0.5,1.0")
    p.add_argument("--gammas", default="1,2,4,8")
    args = p.parse_args()
    import numpy as np
    import torch
    import paper_2511_07421_amd as a3
    from workloads import get_config, make_graph, make_features, degree_ranked_cache, seed_batch

    assert torch.cuda.is_available(), "needs a GPU"
    dev = torch.device("cuda", 0)
    w = get_config(args.workload)
    batches = [int(x) for x in args.batches.split(",")]
    fracs = [float(x) for x in args.cache.split(",")]
    gammas = [float(x) for x in args.gammas.split(",")]
    g = make_graph(w.num_nodes, w.mean_degree, w.d_min, w.d_max, w.a, w.symmetric, w.graph_seed,
                   w.idx_dtype, device=dev)
    full = make_features(w.num_nodes, w.feat_dim, w.feat_dtype, device=dev)
    idx_np = np.int32 if w.idx_dtype == torch.int32 else np.int64
    K, W = args.steps, args.warmup
    st = g.stats()
    print(f"# sweep on `{w.name}`: N={st['num_nodes']:,}, nnz={st['nnz']:,}, fanouts {w.fanouts}, "
          f"{w.row_bytes}-B rows, {K} timed mini-batches per cell (device times from HIP events)")
    print("| batch | cache | gamma | hit rate | input rows | ms sample | ms gather | ms total | "
          "vs gamma=1 | PCIe GB/s | ms per step, 2 in flight | vs gamma=1 |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|")
    for frac in fracs:
        split = degree_ranked_cache(g, full, frac, pin_host=True)
        for batch in batches:
            ctx = a3.Context(batch, w.fanouts, flags=a3.A3_PROFILE)
            cap_rows = batch
            for f in w.fanouts:
                cap_rows *= 1 + f
            cap_rows = min(cap_rows, w.num_nodes)
            out = torch.empty((cap_rows, w.feat_dim), dtype=w.feat_dtype, device=dev)
            out2 = torch.empty_like(out)
            pipe = a3.Pipeline(a3.A3_PIPE_MODE2, 2, batch, w.fanouts)
            seeds = [torch.from_numpy(seed_batch(w.num_nodes, batch, 0, b, dtype=idx_np)).to(dev)
                     for b in range(K + W)]
            base_total = base_piped = None
            for gamma in gammas:
                q = int(round(gamma * 65536))
                hits = rows = 0
                for b in range(K + W):
                    ctx.sample_blocks_begin(g.indptr, g.indices, seeds[b], w.fanouts, split.cache_map, q, b)
                    ctx.gather_input_features(split.feat_dev, split.feat_host, split.cache_map, out)
                    blk = ctx.sample_blocks_end()
                    if b == W - 1:
                        torch.cuda.synchronize()
                        ctx.profile_read(0), ctx.profile_read(1)
                    if b >= W:
                        ids = blk.input_nodes.long()
                        hits += int((split.cache_map[ids] >= 0).sum().item())
                        rows += ids.numel()
                torch.cuda.synchronize()
                ms_s = sum(ctx.profile_read(0)) / K
                ms_g = sum(ctx.profile_read(1)) / K
                total = ms_s + ms_g
                if gamma == gammas[0]:
                    base_total = total
                miss_bytes = (rows - hits) / K * w.row_bytes
                pcie = miss_bytes / (ms_g * 1e-3) / 1e9 if rows > hits else 0.0
                # the same mini-batches with two in flight (Sec. III-B, parallel mode 2: the next
                # mini-batch is sampled beside this one's retrieve, retrieves one at a time): wall time
                outs = (out, out2)
                t0 = 0.0
                for j in range(K + W + 2):
                    if j == W:          # drain the warm-up mini-batches; the K timed ones follow
                        torch.cuda.synchronize()
                        t0 = time.perf_counter()
                    if j >= 2:
                        pipe.wait()
                    if j < K + W:
                        pipe.submit(g.indptr, g.indices, seeds[j], w.fanouts, split.cache_map, q, j,
                                    split.feat_dev, split.feat_host, outs[j % 2])
                torch.cuda.synchronize()
                piped = (time.perf_counter() - t0) * 1e3 / K
                if gamma == gammas[0]:
                    base_piped = piped
                print(f"| {batch} | {frac:.0%} | {gamma:g} | {hits / max(rows, 1):.3f} | {rows // K} | "
                      f"{ms_s:.3f} | {ms_g:.3f} | {total:.3f} | {base_total / total:.2f}x | {pcie:.1f} | "
                      f"{piped:.3f} | {base_piped / piped:.2f}x |", flush=True)
            pipe.close()
            ctx.close()
            del out, out2
        del split


if __name__ == "__main__":
    main()
