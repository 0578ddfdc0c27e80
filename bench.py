#!/usr/bin/env python3
"""Benchmark of the A3GNN mini-batch hot path on one MI355X.

A step is one pass of the whole path over one mini-batch of synthetic input that is already
resident in HBM: a3_sample_blocks_begin/_end (frontier degrees, keyed selection, dedup/relabel
into block CSRs, every hop) and a3_gather_input_features for the input nodes.  Prints ONE JSON
line.  The headline workload is the largest single-GPU configuration (`citation`: 100 M nodes,
1.6 G edges, 8-byte ids, 128 x fp16 rows); the default run also measures `social` and
`copurchase` and reports them under "other_workloads".

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload citation|social|copurchase|tiny]
    python bench.py --sweep      # batch x cache x bias-rate table on the co-purchase graph (markdown)
    python bench.py --policies   # degree-ranked / access-count-ranked / FIFO caches (markdown)
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth
# plain integer ALU peak: 256 CUs x 64 lanes x 2.4 GHz 32-bit lane-operations per second
ALU_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12
# lane-operations the method needs per scanned neighbour slot: a quarter of a Philox4x32-10 block
# (20 32x32->64 multiplies at a quarter of the 32-bit rate = 80, plus 20 three-way xors) and one
# comparison of the draw
OPS_PER_SLOT = (20 * 4 + 20) / 4 + 1
HEADLINE = "citation"
OTHERS = ["social", "copurchase"]
METRIC = "sampled edges/s + feature-gather GB/s (% of HBM peak) per mini-batch, 1 GPU"


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=20)
    p.add_argument("--warmup", type=int, default=5)
    p.add_argument("--workload", default=None,
                   help="measure this workload only (default: %s as the headline, then %s)"
                        % (HEADLINE, ", ".join(OTHERS)))
    p.add_argument("--bias-rate", type=float, default=None, help="gamma (default: the workload's last)")
    p.add_argument("--cache-frac", type=float, default=None)
    p.add_argument("--batch", type=int, default=None)
    p.add_argument("--cpu-seconds", type=float, default=20.0,
                   help="budget of the oracle (CPU baseline) leg; 0 disables it")
    p.add_argument("--row-align", type=int, default=128,
                   help="bytes between row starts of the feature stores and of the output are a "
                        "multiple of this (0: packed rows)")
    p.add_argument("--no-pipelines", action="store_true",
                   help="skip the extra leg that runs the same steps through the stream pipelines")
    p.add_argument("--traffic-bytes", type=float, default=None,
                   help="measured HBM bytes per gather launch (from rocprofv3 --pmc), if known")
    p.add_argument("--pmc-calibration", action="store_true",
                   help="also run plain device copies of 256 MiB (a known size) so that a rocprofv3 "
                        "--pmc run of this command can scale FETCH_SIZE / WRITE_SIZE")
    p.add_argument("--separate-retrieve", action="store_true",
                   help="main leg as a3_sample_blocks_begin + a3_gather_input_features instead of "
                        "a3_sample_gather_begin (which, where rows sit in host memory, retrieves the rows "
                        "of earlier hops on a second stream while later hops are sampled)")
    p.add_argument("--sweep", action="store_true", help="config 4: batch x cache x bias-rate table")
    p.add_argument("--policies", action="store_true", help="cache policies table")
    p.add_argument("--batches", default="256,1024,4096,16384", help="--sweep: batch sizes")
    p.add_argument("--cache", default="0.05,0.2,0.5,1.0", help="--sweep: cache fractions")
    p.add_argument("--gammas", default=None, help="--sweep (default 1,2,4,8) / --policies (default 1,4)")
    p.add_argument("--presample", type=int, default=20, help="--policies: pre-sampled mini-batches")
    return p.parse_args()


def recorded_traffic(workload):
    """HBM bytes per k_gather launch measured with rocprofv3 --pmc (a summary under profiles/)."""
    path = os.path.join(ROOT, "profiles", "%s_gather_pmc.txt" % workload)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1])
    except OSError:
        pass
    return None


def cap_rows_of(w, batch):
    """output rows: at most every node, at most seeds x prod(1 + fanout)"""
    cap = batch
    for f in w.fanouts:
        cap *= 1 + f
    return min(cap, w.num_nodes)


def measure(args, name, headline, legs):
    """One workload: K timed steps, then the legs asked for ("mean", "pipelines", "cpu")."""
    import numpy as np
    import torch
    import paper_2511_07421_amd as a3
    from workloads import (get_config, make_graph, make_features, degree_ranked_cache, padded_rows,
                           seed_batch)

    dev = torch.device("cuda", 0)
    w = get_config(name)
    own = headline or args.workload is not None   # the overrides apply to the workload that was asked for
    gamma = args.bias_rate if (args.bias_rate is not None and own) else w.bias_rates[-1]
    cache_frac = args.cache_frac if (args.cache_frac is not None and own) else w.cache_frac
    batch = (args.batch if own else None) or w.batch
    K, W = args.steps, args.warmup

    t_gen = time.time()
    g = make_graph(w.num_nodes, w.mean_degree, w.d_min, w.d_max, w.a, w.symmetric, w.graph_seed,
                   w.idx_dtype, device=dev)
    full = make_features(w.num_nodes, w.feat_dim, w.feat_dtype, device=dev)
    split = degree_ranked_cache(g, full, cache_frac, pin_host=True, row_align=args.row_align)
    del full
    d_cm = split.cache_map
    idx_np = np.int32 if w.idx_dtype == torch.int32 else np.int64
    seeds = [torch.from_numpy(seed_batch(w.num_nodes, batch, 0, b, dtype=idx_np)).to(dev)
             for b in range(K + W)]
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen
    stats = g.stats()
    ib = stats["idx_bytes"]
    row_bytes = w.row_bytes

    # The timed mini-batches run on a context that brackets only the retrieve with HIP events (the
    # roofline's launch duration); the sampling time comes from a repeat of the same mini-batches
    # on a context that brackets everything.  Each event costs the stream about 4 us: with all
    # five of them a mini-batch of 0.19 ms takes 0.205.
    ctx = a3.Context(batch, w.fanouts, flags=a3.A3_PROFILE_RETRIEVE | a3.A3_STATIC_MAP)
    bias_q16 = int(round(gamma * 65536))
    cap_rows = cap_rows_of(w, batch)
    out = padded_rows(cap_rows, w.feat_dim, w.feat_dtype, dev, args.row_align)
    row_stride = (out.stride(0) if cap_rows > 1 else w.feat_dim) * out.element_size()

    n_edges = n_in = n_in_last = 0
    # a3_sample_gather_begin sends rows ahead only where some may sit in host memory
    parts_ahead = (not args.separate_retrieve and split.feat_host is not None and d_cm is not None
                   and len(w.fanouts) > 1)
    last_ids = None
    last_blocks = None
    slow_paths = {}

    def step(b, timed):
        nonlocal n_edges, n_in, n_in_last, last_ids, last_blocks
        # queue sampling, then the gather of its input nodes (row count taken on the device),
        # then wait for the sampling counts: the host never stalls the GPU between the two
        if not args.separate_retrieve:
            ctx.sample_gather_begin(g.indptr, g.indices, seeds[b], w.fanouts, d_cm, bias_q16, b,
                                    split.feat_dev, split.feat_host, out)
        else:
            ctx.sample_blocks_begin(g.indptr, g.indices, seeds[b], w.fanouts, d_cm, bias_q16, b)
            ctx.gather_input_features(split.feat_dev, split.feat_host, d_cm, out)
        blocks = ctx.sample_blocks_end()
        rows = blocks.n_src[-1]
        assert rows <= cap_rows
        if timed:
            for key, val in ctx.sample_stats().items():
                keep_max = key in ("weight_classes", "launch_plan")
                slow_paths[key] = max(val, slow_paths.get(key, 0)) if keep_max else slow_paths.get(key, 0) + val
            n_edges += sum(blocks.n_edges)
            n_in += rows
            n_in_last += rows - blocks.n_src[-2] if parts_ahead else rows   # rows of the launch behind the sampling
            last_ids = blocks.input_nodes
            last_blocks = blocks
        return blocks

    if args.pmc_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        # the same with the library's own gather kernel on a known volume: ids 0..n-1, no device
        # map, i.e. a plain copy of n rows (read n*row_bytes, write n*row_bytes)
        n_cal = min(100_000, split.n_cached)
        cal_ids = torch.arange(n_cal, dtype=w.idx_dtype, device=dev)
        for _ in range(3):
            ctx.gather_features(split.feat_dev, None, None, cal_ids, out=out[:n_cal])
        torch.cuda.synchronize()
        print("pmc calibration: 3 x 256 MiB device copies, then 3 x identity k_gather of %d rows x %d B"
              % (n_cal, row_bytes), file=sys.stderr)
    for b in range(W):
        step(b, False)
    torch.cuda.synchronize()
    ctx.profile_read(1)   # drop the warm-up calls' timings
    t0 = time.perf_counter()
    for b in range(W, W + K):
        step(b, True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    total_s = t1 - t0
    # device time of each retrieve launch, from HIP events the library records on its stream
    ms_g = ctx.profile_read(1)
    ms_gather = sum(ms_g) * K / len(ms_g)
    ids_l = last_ids.to(torch.int64, copy=True)   # a copy: last_ids is a view of the context's own memory
    # the same mini-batches once more, every call bracketed: the sampling's device time
    ctx.close()
    ctx = a3.Context(batch, w.fanouts, flags=a3.A3_PROFILE | a3.A3_STATIC_MAP)
    for b in range(max(W - 2, 0), W):
        step(b, False)
    torch.cuda.synchronize()
    ctx.profile_read(0), ctx.profile_read(1)
    t2 = time.perf_counter()
    for b in range(W, W + K):
        step(b, False)
    torch.cuda.synchronize()
    repeat_s = time.perf_counter() - t2
    ms_s, ms_g_repeat = ctx.profile_read(0), ctx.profile_read(1)
    assert len(ms_s) == len(ms_g) == min(K, a3.A3_PROFILE_DEPTH)
    ms_sample = sum(ms_s) * K / len(ms_s)
    # hit rate of the last timed batch (outside the timed region)
    hit_rate = int((d_cm[ids_l] >= 0).sum().item()) / ids_l.numel() if ids_l.numel() else 1.0

    # neighbour slots the last timed batch had to draw for (nodes with degree above the fanout)
    scanned_per_hop = []
    for h, f in enumerate(w.fanouts):
        dst = ids_l[:last_blocks.n_dst[h]]
        deg = g.indptr[dst + 1] - g.indptr[dst]
        scanned_per_hop.append(int(deg[deg > f].sum().item()))
    scanned = sum(scanned_per_hop)
    scan_rate = scanned / (ms_sample / K * 1e-3)

    # counters cannot be read from inside this process: the figure comes from the committed
    # rocprofv3 --pmc summary of this same command, and only for the configuration it was taken on
    traffic = args.traffic_bytes if own else None
    if (traffic is None and gamma == w.bias_rates[-1] and cache_frac == w.cache_frac and batch == w.batch
            and args.row_align == 128):
        traffic = recorded_traffic(w.name)

    gather_payload_gbps = n_in_last * row_bytes / (ms_gather * 1e-3) / 1e9
    # per input row: its id, its device-map entry, the row read and the row written
    algo_bytes_per_launch = (n_in_last / K) * (2 * row_bytes + ib + 4)
    gather_avg_s = ms_gather * 1e-3 / K
    achieved = algo_bytes_per_launch / gather_avg_s / 1e9
    result = {
        "metric": METRIC,
        "value": n_edges / total_s,
        "unit": "sampled edges/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": total_s * 1e3 / K,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        # the arithmetic of the path: 32-bit draws (Philox words), 64-bit integer keys; rows are copied
        "dtype": "u32",
        "dtype_note": "u32 draws and u64 integer keys; %d-byte ids; %s rows copied byte for byte"
                      % (ib, str(w.feat_dtype).replace("torch.", "")),
        "data": "synthetic",
        "config": {"workload": w.name, "num_nodes": stats["num_nodes"], "nnz": stats["nnz"],
                   "mean_degree": round(stats["mean_degree"], 2), "max_degree": stats["max_degree"],
                   "idx_bytes": ib, "row_bytes": row_bytes, "batch": batch, "fanouts": w.fanouts,
                   "bias_rate": gamma, "cache_frac": cache_frac, "row_stride_bytes": row_stride,
                   "generate_seconds": round(t_gen, 2)},
        "gather_GBps": gather_payload_gbps,
        "gather_frac_of_hbm_peak": achieved / HBM_PEAK_GBPS,
        "sample_edges_per_s": n_edges / (ms_sample * 1e-3),
        "ms_sample": ms_sample / K,
        "ms_gather": ms_gather / K,
        "ms_sample_note": "from a repeat of the timed mini-batches with every call bracketed by HIP events "
                          "(%.4f ms per step there); the timed region brackets only the retrieve" % (repeat_s * 1e3 / K),
        "ms_sample_median_min": [sorted(ms_s)[len(ms_s) // 2], min(ms_s)],
        "ms_gather_median_min": [sorted(ms_g)[len(ms_g) // 2], min(ms_g)],
        # rows that are not in the HBM cache cross PCIe (zero-copy reads of pinned host memory)
        # (with rows sent ahead the link works during the sampling too: the rate is over the whole step)
        "pcie_GBps": ((n_in / K) * (1.0 - hit_rate) * row_bytes / (total_s / K if parts_ahead else gather_avg_s) / 1e9
                      if hit_rate < 1.0 else 0.0),
        "retrieve": ("rows of earlier hops on a second stream beside the sampling of later hops; ms_gather and "
                     "roofline are the last part's, pcie_GBps is over the whole step" if parts_ahead
                     else "one launch behind the sampling"),
        "rows_behind_sampling_per_step": n_in_last / K,
        "hbm_traffic_GBps": traffic / gather_avg_s / 1e9 if traffic else None,
        "edges_per_step": n_edges / K,
        "input_rows_per_step": n_in / K,
        "cache_hit_rate": hit_rate,
        "scanned_slots_per_step": scanned,
        "scanned_slots_per_hop": scanned_per_hop,
        # nodes of the K timed steps that left the sampler's usual path (a3_sample_stats)
        "slow_path_nodes": slow_paths,
        "roofline_sampling": {"kernel": "k_sample (all hops, with the relabel kernels around it)",
                              "bound": "alu", "achieved": scan_rate * OPS_PER_SLOT / 1e12,
                              "peak": ALU_PEAK_TOPS, "unit": "Tops/s (32-bit integer lane-operations)",
                              "frac": scan_rate * OPS_PER_SLOT / 1e12 / ALU_PEAK_TOPS,
                              "slots_per_s": scan_rate, "ops_per_slot": OPS_PER_SLOT},
        "roofline": {"kernel": "k_gather", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": traffic,
                     "algorithmic_bytes_per_launch": algo_bytes_per_launch,
                     "avg_launch_seconds": gather_avg_s},
    }

    # what this machine's host link gives a plain copy: 256 MiB from pinned host memory to the device,
    # by the runtime's copy engine (outside the timed region; only where rows cross the link)
    if split.feat_host is not None and hit_rate < 1.0:
        n_copy = 256 << 20
        src = torch.empty(n_copy, dtype=torch.uint8, pin_memory=True)
        dst = torch.empty(n_copy, dtype=torch.uint8, device=dev)
        dst.copy_(src, non_blocking=True)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(4):
            dst.copy_(src, non_blocking=True)
        e1.record()
        torch.cuda.synchronize()
        result["pcie_plain_copy_GBps"] = 4 * n_copy / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del src, dst

    # the step after the path: mean aggregation of the gathered rows over the outermost block
    # (a3_block_mean_of_hop), timed by the library's events on a few of the same mini-batches
    if "mean" in legs and w.feat_dtype in (torch.float32, torch.float16):
        H = len(w.fanouts)
        agg_rows = batch
        for f in w.fanouts[:-1]:
            agg_rows *= 1 + f
        agg = padded_rows(min(agg_rows, w.num_nodes), w.feat_dim, w.feat_dtype, dev, args.row_align)
        ctx.profile_read(2)
        m_edges = m_dst = 0
        n_mean = min(K, 10)
        for b in range(W, W + n_mean):
            if not args.separate_retrieve:
                ctx.sample_gather_begin(g.indptr, g.indices, seeds[b], w.fanouts, d_cm, bias_q16, b,
                                        split.feat_dev, split.feat_host, out)
            else:
                ctx.sample_blocks_begin(g.indptr, g.indices, seeds[b], w.fanouts, d_cm, bias_q16, b)
                ctx.gather_input_features(split.feat_dev, split.feat_host, d_cm, out)
            ctx.block_mean_of_hop(H - 1, out, agg)
            blk = ctx.sample_blocks_end()
            m_edges += blk.n_edges[-1]
            m_dst += blk.n_dst[-1]
        torch.cuda.synchronize()
        ms_m = ctx.profile_read(2)
        mean_s = sum(ms_m) / len(ms_m) * 1e-3
        # bytes the aggregation must move through the memory system per launch: one source row
        # and one 4-byte local id per edge, one output row and one 4-byte offset per destination
        mean_bytes = (m_edges * (row_bytes + 4) + m_dst * (row_bytes + 4)) / n_mean
        result["block_mean"] = {"kernel": "k_block_mean (outermost block, rows of the gather)",
                                "bound": "hbm", "achieved": mean_bytes / mean_s / 1e9,
                                "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                "frac": mean_bytes / mean_s / 1e9 / HBM_PEAK_GBPS,
                                "avg_launch_seconds": mean_s, "edges_per_launch": m_edges / n_mean,
                                "dst_per_launch": m_dst / n_mean,
                                "algorithmic_bytes_per_launch": mean_bytes}
        del agg

    if "pipelines" in legs:
        # the same K mini-batches through the scheduling templates of Sec. III-B: n mini-batches in
        # flight on streams of their own (mode 1: whole mini-batches overlap; mode 2: sampling
        # overlaps, the feature retrieve is serialised).  `value` above stays the sequential figure.
        ctx.close()
        ctx = None
        pipes = []
        names = {a3.A3_PIPE_SEQUENTIAL: "sequential", a3.A3_PIPE_MODE1: "mode1", a3.A3_PIPE_MODE2: "mode2"}
        # the last entries add the stage the paper's formulas call "train": a consumer on the
        # caller's stream (the mean aggregation of the outermost block) that works on a finished
        # mini-batch while the workers prepare the next ones
        can_consume = w.feat_dtype in (torch.float32, torch.float16)
        consumer = a3.Context(8, [1]) if can_consume else None
        agg = None
        if can_consume:
            agg_rows = batch
            for f in w.fanouts[:-1]:
                agg_rows *= 1 + f
            agg = padded_rows(min(agg_rows, w.num_nodes), w.feat_dim, w.feat_dtype, dev, args.row_align)
        plans = [(a3.A3_PIPE_SEQUENTIAL, 1, False), (a3.A3_PIPE_MODE1, 2, False), (a3.A3_PIPE_MODE1, 3, False),
                 (a3.A3_PIPE_MODE2, 2, False)]
        if can_consume:
            plans += [(a3.A3_PIPE_SEQUENTIAL, 1, True), (a3.A3_PIPE_MODE1, 3, True)]
        for mode, n_w, consume in plans:
            pipe = a3.Pipeline(mode, n_w, batch, w.fanouts, flags=a3.A3_STATIC_MAP)
            # a worker must not start its next mini-batch (which overwrites its blocks and its
            # row buffer) before the consumer has read the previous one: an event per worker
            worker_streams = [torch.cuda.ExternalStream(pipe.stream(k), device=dev) for k in range(n_w)]
            consumed = [None] * n_w
            outs = [out] + [padded_rows(cap_rows, w.feat_dim, w.feat_dtype, dev, args.row_align)
                            for _ in range(n_w - 1)]
            torch.cuda.synchronize()
            # n_w + W warm-up mini-batches, then the K timed ones of the main leg
            order = [i % (W + K) for i in range(n_w + W)] + list(range(W, W + K))
            first_timed = n_w + W
            p_edges = 0
            t_start = 0.0
            for j in range(len(order) + n_w):
                if j == first_timed:  # everything before is complete; the timed ones start here
                    torch.cuda.synchronize()
                    t_start = time.perf_counter()
                if j >= n_w:
                    blk = pipe.wait()
                    if j - n_w >= first_timed:
                        p_edges += sum(blk.n_edges)
                    if consume:
                        k = (j - n_w) % n_w
                        consumer.block_mean(blk.blk_indptr[-1], blk.blk_indices[-1],
                                            outs[k][: blk.n_src[-1]], out=agg[: blk.n_dst[-1]])
                        consumed[k] = torch.cuda.Event()
                        consumed[k].record()
                if j < len(order):
                    b = order[j]
                    if consumed[j % n_w] is not None:
                        worker_streams[j % n_w].wait_event(consumed[j % n_w])
                    pipe.submit(g.indptr, g.indices, seeds[b], w.fanouts, d_cm, bias_q16, b,
                                split.feat_dev, split.feat_host, outs[j % n_w])
            torch.cuda.synchronize()
            p_s = time.perf_counter() - t_start
            # the same mini-batches, the same edges, and the last of them with the input nodes of the
            # main leg's last one, in the same order (the full-size parity tests compare a pipeline's
            # blocks and rows with the oracle element by element)
            assert p_edges == n_edges
            assert torch.equal(blk.input_nodes.long(), ids_l)
            pipes.append({"mode": names[mode], "workers": n_w, "consumer": "block mean" if consume else None,
                          "ms_per_step": p_s * 1e3 / K, "edges_per_s": p_edges / p_s,
                          "workspace_bytes": pipe.workspace_bytes,
                          "output_bytes": n_w * cap_rows * row_stride})
            pipe.close()
            del outs
        if consumer is not None:
            consumer.close()
        result["pipelines"] = pipes

    if "cpu" in legs and args.cpu_seconds > 0:
        import oracle
        ip_h, ix_h = g.indptr.cpu().numpy(), g.indices.cpu().numpy()
        cm_h = d_cm.cpu().numpy()

        def oracle_rows(ids):
            """the oracle's gather on host copies of only the rows it touches (the whole store of
            `citation` is 25.6 GB), renumbered; returns its seconds"""
            c = cm_h[ids]
            dev_rows, host_rows = np.unique(c[c >= 0]), np.unique(-c[c < 0] - 1)
            fd = split.feat_dev[torch.from_numpy(dev_rows).to(dev)].cpu().numpy() if dev_rows.size else None
            fh = split.feat_host[torch.from_numpy(host_rows)].numpy() if host_rows.size else None
            cm_small = np.zeros_like(c)
            cm_small[c >= 0] = np.searchsorted(dev_rows, c[c >= 0])
            cm_small[c < 0] = -np.searchsorted(host_rows, -c[c < 0] - 1) - 1
            c0 = time.perf_counter()
            oracle.gather_features(fd, fh, cm_small, np.arange(ids.shape[0], dtype=np.int64))
            return time.perf_counter() - c0

        # The oracle as it stands, single-threaded, on a bounded sample of the last timed
        # mini-batch (all its seeds, same rng_seed): its first hop, then as many of its hops as are
        # predicted to fit the budget.  A whole mini-batch of `citation` takes the oracle about two
        # minutes (its parity with the GPU path at full size is the tests' business); its first two
        # hops take about twenty seconds.
        H = len(w.fanouts)
        seeds_host = {}

        def oracle_run(b, hops):
            if b not in seeds_host:
                seeds_host[b] = seeds[b].cpu().numpy()
            c0 = time.perf_counter()
            ob = oracle.sample_blocks(ip_h, ix_h, seeds_host[b], w.fanouts[:hops], cm_h, bias_q16, b)
            return ob, time.perf_counter() - c0

        b_last = W + K - 1
        ob, dt = oracle_run(b_last, 1)
        dg = oracle_rows(ob.input_nodes.astype(np.int64))
        spent, best = dt + dg, (1, ob, dt, dg)
        # the oracle scans five to six million neighbour slots a second on one core, and the slots
        # that each hop scans are known from the GPU's blocks: as many hops as twelve million slots
        # per second of budget allow (so the run takes up to about twice the budget; the default
        # budget of 20 s admits the first two hops of `citation`, 204 M slots, and all of the others)
        hops = 1
        while hops < H and sum(scanned_per_hop[:hops + 1]) <= 12e6 * args.cpu_seconds:
            hops += 1
        if hops > 1:
            ob, dt = oracle_run(b_last, hops)
            dg = oracle_rows(ob.input_nodes.astype(np.int64))
            spent += dt + dg
            best = (hops, ob, dt, dg)
        hops, ob, dt, dg = best
        result["cpu_baseline"] = {
            "value": sum(ob.n_edges) / (dt + dg), "unit": "sampled edges/s", "cores": 1, "kind": "oracle",
            "sample": "the first %d of %d hops of the last timed mini-batch of workload %s (all its seeds, same "
                      "rng_seed), sampling + gather of that run's input rows: %d edges in %.1f s; %.1f s of CPU "
                      "work with the one-hop run before it" % (hops, H, w.name, sum(ob.n_edges), dt + dg, spent),
            "hops": hops, "edges": sum(ob.n_edges),
            "gather_GBps": ob.n_src[-1] * row_bytes / max(dg, 1e-9) / 1e9,
            "ms_sample": dt * 1e3, "ms_gather": dg * 1e3,
        }
        # the unchanged oracle over independent mini-batches, one per thread, on the host's cores
        # (its C code runs outside the interpreter lock), the same number of hops each
        n_thr = min(16, os.cpu_count() or 1, K - 1)
        if n_thr > 1:
            from concurrent.futures import ThreadPoolExecutor
            todo = list(range(W, W + n_thr))
            for b in todo:
                seeds_host[b] = seeds[b].cpu().numpy()
            c0 = time.perf_counter()
            with ThreadPoolExecutor(n_thr) as pool:
                a_edges = sum(sum(o.n_edges) for o, _ in pool.map(lambda b: oracle_run(b, hops), todo))
            a_s = time.perf_counter() - c0
            model = ""
            try:
                with open("/proc/cpuinfo") as f:
                    model = next((ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")), "")
            except OSError:
                pass
            result["cpu_baseline_all_cores"] = {
                "value": a_edges / a_s, "unit": "sampled edges/s (sampling + reindex, no gather)",
                "cores": n_thr, "kind": "oracle",
                "sample": "the first %d hops of %d further timed mini-batches, one per thread, %.1f s wall"
                          % (hops, n_thr, a_s),
                "cpu_model": model,
            }
        # whole timed mini-batches on the library's own multi-threaded host sampler (the paper's
        # "Sampling Device = CPU, Workers = n"): sampling + reindex only, bit-identical blocks
        n_workers = min(16, os.cpu_count() or 1)
        cpu = a3.CpuSampler(n_workers)
        c_edges, c_s, c_done = 0, 0.0, 0
        while c_s < args.cpu_seconds / 4 and c_done < K:
            s_h = seeds[W + c_done].cpu().numpy()
            c0 = time.perf_counter()
            cb = cpu.sample_blocks(ip_h, ix_h, s_h, w.fanouts, cm_h, bias_q16, W + c_done)
            c_s += time.perf_counter() - c0
            c_edges += sum(cb.n_edges)
            c_done += 1
        cpu.close()
        result["cpu_sampler"] = {
            "value": c_edges / c_s, "unit": "sampled edges/s (sampling + reindex, no gather)",
            "cores": n_workers, "kind": "a3cpu_sample_blocks, the library's multi-threaded host sampler",
            "sample": "%d of the timed mini-batches, %.1f s" % (c_done, c_s),
            "ms_sample": c_s * 1e3 / c_done,
        }
    if ctx is not None:
        ctx.close()
    return result


def run_sweep(args):
    """Batch / cache / bias-rate sweep on the co-purchase-style graph.  Shows where
    locality-aware sampling pays off (Sec. II-B Motivation 2, Sec. IV-C ablation): for every batch
    size x HBM cache fraction x bias rate it reports the cache hit rate of the input nodes, the
    number of input rows, the device time of sampling and of the feature gather (HBM rows +
    pinned-host rows over PCIe) as separate calls, the wall time per mini-batch as one unit
    (a3_sample_gather_begin: rows of earlier hops cross the link during the sampling of later
    hops), and with two mini-batches in flight (parallel mode 2: sampling beside the previous
    retrieve).  Markdown table; one graph."""
    import numpy as np
    import torch
    import paper_2511_07421_amd as a3
    from workloads import get_config, make_graph, make_features, degree_ranked_cache, padded_rows, seed_batch

    dev = torch.device("cuda", 0)
    w = get_config(args.workload or "copurchase")
    batches = [int(x) for x in args.batches.split(",")]
    fracs = [float(x) for x in args.cache.split(",")]
    gammas = [float(x) for x in (args.gammas or "1,2,4,8").split(",")]
    g = make_graph(w.num_nodes, w.mean_degree, w.d_min, w.d_max, w.a, w.symmetric, w.graph_seed,
                   w.idx_dtype, device=dev)
    full = make_features(w.num_nodes, w.feat_dim, w.feat_dtype, device=dev)
    idx_np = np.int32 if w.idx_dtype == torch.int32 else np.int64
    K, W = args.steps, min(args.warmup, 2)
    st = g.stats()
    print(f"# sweep on `{w.name}`: N={st['num_nodes']:,}, nnz={st['nnz']:,}, fanouts {w.fanouts}, "
          f"{w.row_bytes}-B rows, {K} timed mini-batches per cell (device times from HIP events)")
    print("| batch | cache | gamma | hit rate | input rows | ms sample | ms gather | ms total | "
          "vs gamma=1 | PCIe GB/s | ms per step, one unit | ms per step, 2 in flight | vs gamma=1 |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    for frac in fracs:
        split = degree_ranked_cache(g, full, frac, pin_host=True, row_align=args.row_align)
        for batch in batches:
            ctx = a3.Context(batch, w.fanouts, flags=a3.A3_PROFILE | a3.A3_STATIC_MAP)
            cap_rows = cap_rows_of(w, batch)
            out = padded_rows(cap_rows, w.feat_dim, w.feat_dtype, dev, args.row_align)
            out2 = padded_rows(cap_rows, w.feat_dim, w.feat_dtype, dev, args.row_align)
            pipe = a3.Pipeline(a3.A3_PIPE_MODE2, 2, batch, w.fanouts, flags=a3.A3_STATIC_MAP)
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
                # the same mini-batches through a3_sample_gather_begin (where rows sit in host memory,
                # those of earlier hops cross the link while later hops are sampled): wall time
                for b in range(K + W):
                    if b == W:
                        torch.cuda.synchronize()
                        t0 = time.perf_counter()
                    ctx.sample_gather_begin(g.indptr, g.indices, seeds[b], w.fanouts, split.cache_map, q, b,
                                            split.feat_dev, split.feat_host, out)
                    ctx.sample_blocks_end()
                torch.cuda.synchronize()
                unit = (time.perf_counter() - t0) * 1e3 / K
                ctx.profile_read(0), ctx.profile_read(1)
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
                      f"{unit:.3f} | {piped:.3f} | {base_piped / piped:.2f}x |", flush=True)
            pipe.close()
            ctx.close()
            del out, out2
        del split


def run_policies(args):
    """Cache policies on the co-purchase-style graph: hit rate and step time of the static fill
    ranked by degree (the input generators' default), the static fill ranked by access count over
    pre-sampled mini-batches (a3_cache_count_accesses + a3_cache_rank; Sec. IV-C fills the cache
    with the nodes accessed most often), and a FIFO dynamic cache that starts empty (a3_cache_fifo_update_static;
    Sec. II-B), each under uniform and locality-aware sampling.  Markdown table."""
    import numpy as np
    import torch
    import paper_2511_07421_amd as a3
    from workloads import get_config, make_graph, make_features, degree_ranked_cache, seed_batch

    dev = torch.device("cuda", 0)
    w = get_config(args.workload or "copurchase")
    cache_frac = args.cache_frac if args.cache_frac is not None else w.cache_frac
    K = args.steps
    g = make_graph(w.num_nodes, w.mean_degree, w.d_min, w.d_max, w.a, w.symmetric, w.graph_seed,
                   w.idx_dtype, device=dev)
    full = make_features(w.num_nodes, w.feat_dim, w.feat_dtype, device=dev)
    N = w.num_nodes
    n_cached = int(np.ceil(cache_frac * N))
    idx_np = np.int32 if w.idx_dtype == torch.int32 else np.int64
    seeds = [torch.from_numpy(seed_batch(N, w.batch, 0, b, dtype=idx_np)).to(dev)
             for b in range(K + args.presample)]
    ctx = a3.Context(w.batch, w.fanouts, flags=a3.A3_PROFILE)
    rows = torch.empty((cap_rows_of(w, w.batch), w.feat_dim), dtype=w.feat_dtype, device=dev)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def host_rows(order_rest):
        host = torch.empty((order_rest.shape[0], w.feat_dim), dtype=w.feat_dtype, pin_memory=True)
        step = 1 << 20
        for r0 in range(0, order_rest.shape[0], step):
            host[r0:r0 + step] = full[order_rest[r0:r0 + step].long()].cpu()
        return host

    def second_launch_nodes(ctx, blk):
        """frontier nodes of a weighted call that its fast sampling launches could not decide, as a
        share of all its frontier nodes (under the single-launch plan: all of them)"""
        st = ctx.sample_stats()
        if st["launch_plan"] == 0:
            return 0.0
        if st["launch_plan"] == 2:
            return 1.0
        return (st["deferred_wide_nodes"] + st["deferred_hubs"]) / max(sum(blk.n_dst), 1)

    def run_static(cache_map, feat_dev, feat_host, gamma):
        q = int(gamma * 65536)
        hits = n_in = left = 0
        ctx.profile_read(0), ctx.profile_read(1)
        for b in range(args.presample, args.presample + K):
            ctx.sample_blocks_begin(g.indptr, g.indices, seeds[b], w.fanouts, cache_map, q, b)
            ctx.gather_input_features(feat_dev, feat_host, cache_map, rows)
            blk = ctx.sample_blocks_end()
            left += second_launch_nodes(ctx, blk)
            ids = blk.input_nodes.long()
            hits += int((cache_map[ids] >= 0).sum().item())
            n_in += ids.numel()
        torch.cuda.synchronize()
        return hits / n_in, n_in / K, sum(ctx.profile_read(0)) / K, sum(ctx.profile_read(1)) / K, left / K

    print(f"# cache policies on `{w.name}`: N={N:,}, {w.row_bytes}-B rows, cache {cache_frac:.0%} = {n_cached:,} rows, "
          f"batch {w.batch}, fanouts {w.fanouts}, {K} mini-batches per row (device times from HIP events)")
    print("| policy | gamma | hit rate | input rows | nodes sampled by the slow launch | ms sample | ms gather | ms policy | ms total |")
    print("|---|---|---|---|---|---|---|---|---|")
    gammas = [float(x) for x in (args.gammas or "1,4").split(",")]
    # 1. degree-ranked static fill
    split = degree_ranked_cache(g, full, cache_frac, pin_host=True)
    for gamma in gammas:
        h, n, ms_s, ms_g, left = run_static(split.cache_map, split.feat_dev, split.feat_host, gamma)
        print(f"| static, by degree | {gamma:g} | {h:.3f} | {n:.0f} | {left:.1%} | {ms_s:.3f} | {ms_g:.3f} | - | {ms_s + ms_g:.3f} |", flush=True)
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
        h, n, ms_s, ms_g, left = run_static(cache_map, feat_dev, feat_host, gamma)
        print(f"| static, by access count ({args.presample} pre-sampled batches, set-up {setup_ms:.1f} ms on the GPU) | {gamma:g} | "
              f"{h:.3f} | {n:.0f} | {left:.1%} | {ms_s:.3f} | {ms_g:.3f} | - | {ms_s + ms_g:.3f} |", flush=True)
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
        hits = n_in = left = 0
        first_hit = last_hit = 0.0
        ms_pol = 0.0
        for b in range(args.presample, args.presample + K):
            ctx.sample_blocks_begin(g.indptr, g.indices, seeds[b], w.fanouts, cm, q, b)
            ctx.gather_input_features(cache, host_all, cm, rows)
            blk = ctx.sample_blocks_end()
            left += second_launch_nodes(ctx, blk)
            ids = blk.input_nodes.long()
            hb = int((cm[ids] >= 0).sum().item())   # judged before the update
            ev0.record()
            ctx.cache_fifo_update(cm, owner, state, cache, rows, static_scratch=True)
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
              f"{hits / n_in:.3f} | {n_in / K:.0f} | {left / K:.1%} | {ms_s:.3f} | {ms_g:.3f} | {ms_pol / K:.3f} | "
              f"{ms_s + ms_g + ms_pol / K:.3f} |", flush=True)
    ctx.close()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2511_07421_amd as a3

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if not os.path.exists(a3.library_path()):
        print("bench.py: HIP library not built (run __graft_entry__.build())", file=sys.stderr)
        sys.exit(2)
    if args.sweep:
        return run_sweep(args)
    if args.policies:
        return run_policies(args)
    legs = {"mean", "cpu"} | (set() if args.no_pipelines else {"pipelines"})
    result = measure(args, args.workload or HEADLINE, True, legs)
    if args.workload is None:
        # the other single-GPU configurations, each at its own headline setting (copurchase with
        # locality-aware sampling, gamma = 4), without the oracle leg
        others = {}
        for name in OTHERS:
            torch.cuda.empty_cache()
            r = measure(args, name, False, legs - {"cpu"})
            for k in ("metric", "n_gpus", "higher_is_better", "scaling", "vs_baseline", "data", "steps", "warmup"):
                r.pop(k, None)
            others[name] = r
        result["other_workloads"] = others
    print(json.dumps(result))


if __name__ == "__main__":
    main()
