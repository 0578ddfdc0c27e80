#!/usr/bin/env python3
"""Cache policies on the co-purchase-style graph (one MI355X): hit rate and step time of

  * the static fill ranked by degree (the input generators' default),
  * the static fill ranked by access count over pre-sampled mini-batches
    (a3_cache_count_accesses + a3_cache_rank; paper Sec. IV-C: "most frequently accessed nodes"),
  * a FIFO dynamic cache that starts empty (a3_cache_fifo_update; Sec. II-B),

each under uniform (gamma = 1) and locality-aware (gamma = 4) sampling.  Prints a markdown table.

    python bench_policies.py [--workload copurchase] [--cache-frac 0.2] [--steps 30] [--presample 20]
"""
import argparse
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    p = argparse.ArgumentParser()
    p.add_argument("--workload", default="copurchase")
    p.add_argument("--cache-frac", type=float, default=0.2)
    p.add_argument("--steps", type=int, default=30)
    p.add_argument("--presample", type=int, default=20)
    p.add_argument("--gammas", default="1,4")
    args = p.parse_args()
    import numpy as np
    import torch
    import paper_2511_07421_amd as a3
    from workloads import get_config, make_graph, make_features, degree_ranked_cache, seed_batch

    assert torch.cuda.is_available(), "needs a GPU"
    dev = torch.device("cuda", 0)
    w = get_config(args.workload)
    K = args.steps
    g = make_graph(w.num_nodes, w.mean_degree, w.d_min, w.d_max, w.a, w.symmetric, w.graph_seed,
                   w.idx_dtype, device=dev)
    full = make_features(w.num_nodes, w.feat_dim, w.feat_dtype, device=dev)
    N = w.num_nodes
    n_cached = int(np.ceil(args.cache_frac * N))
    idx_np = np.int32 if w.idx_dtype == torch.int32 else np.int64
    seeds = [torch.from_numpy(seed_batch(N, w.batch, 0, b, dtype=idx_np)).to(dev)
             for b in range(K + args.presample)]
    ctx = a3.Context(w.batch, w.fanouts, flags=a3.A3_PROFILE)
    cap_rows = w.batch
    for f in w.fanouts:
        cap_rows *= 1 + f
    rows = torch.empty((min(cap_rows, N), w.feat_dim), dtype=w.feat_dtype, device=dev)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def host_rows(order_rest):
        host = torch.empty((order_rest.shape[0], w.feat_dim), dtype=w.feat_dtype, pin_memory=True)
        step = 1 << 20
        for r0 in range(0, order_rest.shape[0], step):
            host[r0:r0 + step] = full[order_rest[r0:r0 + step].long()].cpu()
        return host

    def run_static(cache_map, feat_dev, feat_host, gamma):
        q = int(gamma * 65536)
        hits = n_in = 0
        ctx.profile_read(0), ctx.profile_read(1)
        for b in range(args.presample, args.presample + K):
            ctx.sample_blocks_begin(g.indptr, g.indices, seeds[b], w.fanouts, cache_map, q, b)
            ctx.gather_input_features(feat_dev, feat_host, cache_map, rows)
            blk = ctx.sample_blocks_end()
            ids = blk.input_nodes.long()
            hits += int((cache_map[ids] >= 0).sum().item())
            n_in += ids.numel()
        torch.cuda.synchronize()
        return hits / n_in, n_in / K, sum(ctx.profile_read(0)) / K, sum(ctx.profile_read(1)) / K

    print(f"# cache policies on `{w.name}`: N={N:,}, {w.row_bytes}-B rows, cache {args.cache_frac:.0%} = {n_cached:,} rows, "
          f"batch {w.batch}, fanouts {w.fanouts}, {K} mini-batches per row (device times from HIP events)")
    print("| policy | gamma | hit rate | input rows | ms sample | ms gather | ms policy | ms total |")
    print("|---|---|---|---|---|---|---|---|")
    gammas = [float(x) for x in args.gammas.split(",")]
    # 1. degree-ranked static fill
    split = degree_ranked_cache(g, full, args.cache_frac, pin_host=True)
    for gamma in gammas:
        h, n, ms_s, ms_g = run_static(split.cache_map, split.feat_dev, split.feat_host, gamma)
        print(f"| static, by degree | {gamma:g} | {h:.3f} | {n:.0f} | {ms_s:.3f} | {ms_g:.3f} | - | {ms_s + ms_g:.3f} |", flush=True)
    del split
    # 2. access-count-ranked static fill: pre-sample, count, rank, build the two stores by gathers
    counts = torch.zeros(N, dtype=torch.int32, device=dev)
    ev0.record()
    for b in range(args.presample):
        ctx.sample_blocks_begin(g.indptr, g.indices, seeds[b], w.fanouts, None, 65536, b)
        ctx.cache_count_accesses(counts)
        ctx.sample_blocks_end()
    cache_map, order = ctx.cache_rank(counts, n_cached)
    feat_dev = ctx.gather_features(full, None, None, order[:n_cached].contiguous())
    ev1.record()
    torch.cuda.synchronize()
    setup_ms = ev0.elapsed_time(ev1)
    feat_host = host_rows(order[n_cached:])
    for gamma in gammas:
        h, n, ms_s, ms_g = run_static(cache_map, feat_dev, feat_host, gamma)
        print(f"| static, by access count ({args.presample} pre-sampled batches, set-up {setup_ms:.1f} ms on the GPU) | {gamma:g} | "
              f"{h:.3f} | {n:.0f} | {ms_s:.3f} | {ms_g:.3f} | - | {ms_s + ms_g:.3f} |", flush=True)
    del feat_dev, feat_host, cache_map, order
    # 3. FIFO dynamic cache from empty; the host store holds every row
    host_all = host_rows(torch.arange(N, device=dev))
    for gamma in gammas:
        q = int(gamma * 65536)
        cm = -torch.arange(N, dtype=torch.int32, device=dev) - 1
        owner = torch.full((n_cached,), -1, dtype=torch.int32, device=dev)
        state = torch.zeros(4, dtype=torch.int32, device=dev)
        cache = torch.zeros((n_cached, w.feat_dim), dtype=w.feat_dtype, device=dev)
        ctx.profile_read(0), ctx.profile_read(1)
        hits = n_in = 0
        first_hit = last_hit = 0.0
        ms_pol = 0.0
        for b in range(args.presample, args.presample + K):
            ctx.sample_blocks_begin(g.indptr, g.indices, seeds[b], w.fanouts, cm, q, b)
            ctx.gather_input_features(cache, host_all, cm, rows)
            blk = ctx.sample_blocks_end()
            ids = blk.input_nodes.long()
            hb = int((cm[ids] >= 0).sum().item())   # judged before the update
            ev0.record()
            ctx.cache_fifo_update(cm, owner, state, cache, rows)
            ev1.record()
            torch.cuda.synchronize()
            ms_pol += ev0.elapsed_time(ev1)
            hits += hb
            n_in += ids.numel()
            if b == args.presample + 1:
                first_hit = hb / ids.numel()
            last_hit = hb / ids.numel()
        ms_s, ms_g = sum(ctx.profile_read(0)) / K, sum(ctx.profile_read(1)) / K
        print(f"| FIFO, from empty (hit rate of batch 2: {first_hit:.3f}, of the last: {last_hit:.3f}) | {gamma:g} | "
              f"{hits / n_in:.3f} | {n_in / K:.0f} | {ms_s:.3f} | {ms_g:.3f} | {ms_pol / K:.3f} | "
              f"{ms_s + ms_g + ms_pol / K:.3f} |", flush=True)
    ctx.close()


if __name__ == "__main__":
    main()
