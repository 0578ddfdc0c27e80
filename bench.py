#!/usr/bin/env python3
"""Benchmark of the A3GNN mini-batch hot path on one MI355X.

A step is one pass of the whole path over one mini-batch of synthetic input that is already
resident in HBM: a3_sample_blocks_begin/_end (frontier degrees, keyed selection, dedup/relabel
into block CSRs, every hop) and a3_gather_input_features for the input nodes.  Prints ONE JSON
line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload social|copurchase|citation|tiny]
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


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=40)
    p.add_argument("--warmup", type=int, default=5)
    p.add_argument("--workload", default="social")
    p.add_argument("--bias-rate", type=float, default=None, help="gamma (default: the workload's first)")
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


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2511_07421_amd as a3
    from workloads import (get_config, make_graph, make_features, degree_ranked_cache, padded_rows,
                           seed_batch)

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if not os.path.exists(a3.library_path()):
        print("bench.py: HIP library not built (run __graft_entry__.build())", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda", 0)
    w = get_config(args.workload)
    gamma = args.bias_rate if args.bias_rate is not None else w.bias_rates[-1]
    cache_frac = args.cache_frac if args.cache_frac is not None else w.cache_frac
    batch = args.batch or w.batch
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

    ctx = a3.Context(batch, w.fanouts, flags=a3.A3_PROFILE)
    bias_q16 = int(round(gamma * 65536))
    # output rows: at most every node, at most seeds x prod(1 + fanout)
    cap_rows = batch
    for f in w.fanouts:
        cap_rows = cap_rows * (1 + f)
    cap_rows = min(cap_rows, w.num_nodes)
    out = padded_rows(cap_rows, w.feat_dim, w.feat_dtype, dev, args.row_align)
    row_stride = (out.stride(0) if cap_rows > 1 else w.feat_dim) * out.element_size()

    n_edges = n_in = 0
    last_ids = None
    last_blocks = None

    def step(b, timed):
        nonlocal n_edges, n_in, last_ids, last_blocks
        # queue sampling, then the gather of its input nodes (row count taken on the device),
        # then wait for the sampling counts: the host never stalls the GPU between the two
        ctx.sample_blocks_begin(g.indptr, g.indices, seeds[b], w.fanouts, d_cm, bias_q16, b)
        ctx.gather_input_features(split.feat_dev, split.feat_host, d_cm, out)
        blocks = ctx.sample_blocks_end()
        rows = blocks.n_src[-1]
        assert rows <= cap_rows
        if timed:
            n_edges += sum(blocks.n_edges)
            n_in += rows
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
    ctx.profile_read(0), ctx.profile_read(1)   # drop the warm-up calls' timings
    t0 = time.perf_counter()
    for b in range(W, W + K):
        step(b, True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    total_s = t1 - t0
    # device time of each call's kernels, from HIP events the library records on its stream
    ms_s, ms_g = ctx.profile_read(0), ctx.profile_read(1)
    assert len(ms_s) == len(ms_g) == min(K, a3.A3_PROFILE_DEPTH)
    ms_sample = sum(ms_s) * K / len(ms_s)
    ms_gather = sum(ms_g) * K / len(ms_g)
    # hit rate of the last timed batch (outside the timed region)
    ids_l = last_ids.long()
    hit_rate = int((d_cm[ids_l] >= 0).sum().item()) / ids_l.numel() if ids_l.numel() else 1.0

    # neighbour slots the last timed batch had to draw for (nodes with degree above the fanout)
    scanned = 0
    for h, f in enumerate(w.fanouts):
        dst = ids_l[:last_blocks.n_dst[h]]
        deg = g.indptr[dst + 1] - g.indptr[dst]
        scanned += int(deg[deg > f].sum().item())
    scan_rate = scanned / (ms_sample / K * 1e-3)

    # counters cannot be read from inside this process: the figure comes from the committed
    # rocprofv3 --pmc summary of this same command, and only for the configuration it was taken on
    traffic = args.traffic_bytes
    if (traffic is None and args.batch is None and args.cache_frac is None and args.bias_rate is None
            and args.row_align == 128):
        traffic = recorded_traffic(w.name)

    gather_payload_gbps = n_in * row_bytes / (ms_gather * 1e-3) / 1e9
    algo_bytes_per_launch = (n_in / K) * (2 * row_bytes + ib + 4)
    gather_avg_s = ms_gather * 1e-3 / K
    achieved = algo_bytes_per_launch / gather_avg_s / 1e9
    result = {
        "metric": "sampled edges/s + feature-gather GB/s (% of HBM peak) per mini-batch, 1 GPU",
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
        "ms_sample_median_min": [sorted(ms_s)[len(ms_s) // 2], min(ms_s)],
        "ms_gather_median_min": [sorted(ms_g)[len(ms_g) // 2], min(ms_g)],
        # rows that are not in the HBM cache cross PCIe (zero-copy reads of pinned host memory)
        "pcie_GBps": (n_in / K) * (1.0 - hit_rate) * row_bytes / gather_avg_s / 1e9 if hit_rate < 1.0 else 0.0,
        "hbm_traffic_GBps": traffic / gather_avg_s / 1e9 if traffic else None,
        "edges_per_step": n_edges / K,
        "input_rows_per_step": n_in / K,
        "cache_hit_rate": hit_rate,
        "scanned_slots_per_step": scanned,
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
    if w.feat_dtype in (torch.float32, torch.float16):
        H = len(w.fanouts)
        agg_rows = batch
        for f in w.fanouts[:-1]:
            agg_rows *= 1 + f
        agg = padded_rows(min(agg_rows, w.num_nodes), w.feat_dim, w.feat_dtype, dev, args.row_align)
        ctx.profile_read(2)
        m_edges = m_dst = 0
        n_mean = min(K, 10)
        for b in range(W, W + n_mean):
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

    if not args.no_pipelines:
        # the same K mini-batches through the scheduling templates of Sec. III-B: n mini-batches in
        # flight on streams of their own (mode 1: whole mini-batches overlap; mode 2: sampling
        # overlaps, the feature retrieve is serialised).  `value` above stays the sequential figure.
        ctx.close()
        pipes = []
        names = {a3.A3_PIPE_SEQUENTIAL: "sequential", a3.A3_PIPE_MODE1: "mode1", a3.A3_PIPE_MODE2: "mode2"}
        # the last entry adds the stage the paper's formulas call "train": a consumer on the
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
                 (a3.A3_PIPE_MODE2, 2, False), (a3.A3_PIPE_MODE2, 3, False)]
        if can_consume:
            plans += [(a3.A3_PIPE_SEQUENTIAL, 1, True), (a3.A3_PIPE_MODE1, 3, True)]
        for mode, n_w, consume in plans:
            pipe = a3.Pipeline(mode, n_w, batch, w.fanouts)
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
            assert p_edges == n_edges  # the same mini-batches, the same edges
            pipes.append({"mode": names[mode], "workers": n_w, "consumer": "block mean" if consume else None,
                          "ms_per_step": p_s * 1e3 / K, "edges_per_s": p_edges / p_s,
                          "workspace_bytes": pipe.workspace_bytes,
                          "output_bytes": n_w * cap_rows * row_stride})
            pipe.close()
            del outs
        if consumer is not None:
            consumer.close()
        result["pipelines"] = pipes

    if args.cpu_seconds > 0:
        import oracle
        ip_h, ix_h = g.indptr.cpu().numpy(), g.indices.cpu().numpy()
        cm_h = d_cm.cpu().numpy()
        fd_h = None if split.feat_dev is None else split.feat_dev.cpu().numpy()
        fh_h = None if split.feat_host is None else split.feat_host.numpy()
        spent, done, o_edges, o_rows, o_sample, o_gather = 0.0, 0, 0, 0, 0.0, 0.0
        while spent < args.cpu_seconds and done < K:
            s_h = seeds[W + done].cpu().numpy()
            c0 = time.perf_counter()
            ob = oracle.sample_blocks(ip_h, ix_h, s_h, w.fanouts, cm_h, bias_q16, W + done)
            c1 = time.perf_counter()
            oracle.gather_features(fd_h, fh_h, cm_h, ob.input_nodes.astype(idx_np))
            c2 = time.perf_counter()
            o_edges += sum(ob.n_edges)
            o_rows += ob.n_src[-1]
            o_sample += c1 - c0
            o_gather += c2 - c1
            spent += c2 - c0
            done += 1
        result["cpu_baseline"] = {
            "value": o_edges / spent, "unit": "sampled edges/s", "cores": 1, "kind": "oracle",
            "sample": "%d of the timed mini-batches of workload %s (same seeds, same rng_seed), "
                      "%.1f s of CPU work" % (done, w.name, spent),
            "gather_GBps": o_rows * row_bytes / max(o_gather, 1e-9) / 1e9,
            "ms_sample": o_sample * 1e3 / done, "ms_gather": o_gather * 1e3 / done,
        }
        # the unchanged oracle over independent mini-batches, one per thread, on the host's cores
        # (its C code runs outside the interpreter lock); skipped where one mini-batch alone
        # outlasts the CPU budget
        n_thr = min(16, os.cpu_count() or 1, K - done)
        if n_thr > 1 and spent / done <= args.cpu_seconds:
            from concurrent.futures import ThreadPoolExecutor

            def one(b):
                ob = oracle.sample_blocks(ip_h, ix_h, seeds_h[b], w.fanouts, cm_h, bias_q16, b)
                oracle.gather_features(fd_h, fh_h, cm_h, ob.input_nodes.astype(idx_np))
                return sum(ob.n_edges)

            seeds_h = {b: seeds[b].cpu().numpy() for b in range(W + done, W + done + n_thr)}
            c0 = time.perf_counter()
            with ThreadPoolExecutor(n_thr) as pool:
                a_edges = sum(pool.map(one, sorted(seeds_h)))
            a_s = time.perf_counter() - c0
            model = ""
            try:
                with open("/proc/cpuinfo") as f:
                    model = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), "")
            except OSError:
                pass
            result["cpu_baseline_all_cores"] = {
                "value": a_edges / a_s, "unit": "sampled edges/s", "cores": n_thr, "kind": "oracle",
                "sample": "%d further timed mini-batches, one per thread, %.1f s wall" % (n_thr, a_s),
                "cpu_model": model,
            }
        # the same mini-batches on the library's own multi-threaded host sampler (the paper's
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
    ctx.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
