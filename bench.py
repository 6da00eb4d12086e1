#!/usr/bin/env python3
"""Mini-batch generation benchmark on one MI355X.

A step is one pass of the whole hot path over one mini-batch: L-hop neighbour
sampling into blocks, feature gather through the HBM cache (misses read from
pinned host memory), and the chain of mean aggregations, on the "medium"
workload (Reddit-shaped synthetic power-law graph, 602-dim fp32 features,
fanouts [25, 10], 1,024 seeds, top 30 % of nodes by degree cached in HBM).
Inputs are resident (graph and cache in HBM, features in pinned host memory)
before the timed region starts.

Prints one JSON line.  `value` = sampled edges per second over the timed,
pipelined region (`ms_per_step` = its time per mini-batch); `roofline` = the
hit-gather kernel against the HBM peak (algorithmic bytes per launch over its
average duration by HIP events, `traffic` = hardware-counter bytes per launch
read from the profile summary); `roofline_host_link` = the miss-gather kernel
against the host link; `cpu_baseline` = the CPU oracle on a sample of the same
mini-batches; `stage_us_per_step` and `kernels` = per-kernel times from a second
pass that runs one mini-batch at a time; the remaining objects report the
optional paths (backward, weighted, layer-wise) measured on the same blocks.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
HOST_LINK_PEAK_GBPS = 64.0      # PCIe Gen5 x16, one direction, nominal


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="medium")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the graph (debugging only)")
    ap.add_argument("--cache-pct", type=int, default=None)
    ap.add_argument("--cache-policy", choices=["top", "sampled", "walk", "walk-sampled"], default="top",
                    help="how the cache is filled: top degree (the workloads' definition), drawn in proportion "
                         "to degree (paper Eq. 13), or by random-walk scores from the training set (Eq. 14-15)")
    ap.add_argument("--in-flight", type=int, default=3, help="mini-batches in flight (contexts x streams)")
    ap.add_argument("--miss-inflight-kb", type=int, default=None, help="KiB of host reads the miss gather keeps outstanding")
    ap.add_argument("--dedup", choices=["bitmap", "hash"], default="bitmap",
                    help="frontier dedup: node-indexed bitmap and position table (default) or hash table and sort")
    ap.add_argument("--prioritise-cache", action="store_true",
                    help="cache-prioritised neighbour sampling: a row's cached neighbours are drawn first "
                         "(another sampling distribution than the workloads define; for comparison)")
    ap.add_argument("--graph", action="store_true",
                    help="record each in-flight slot's step (sample, gather, aggregate) into a HIP graph once and "
                         "replay it in the timed region (seeds and sampling seed are rewritten in device buffers)")
    ap.add_argument("--heavy-degree", type=int, default=None, help="degree above which a workgroup samples a row")
    ap.add_argument("--device-row-multiple", type=int, default=None,
                    help="bytes the rows kept in HBM are padded to a multiple of (default: synth.aligned_row_stride)")
    ap.add_argument("--cpu-batches", type=int, default=None, help="oracle batches for the CPU baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-copy", action="store_true",
                    help="also launch one plain 1 GiB read + 1 GiB write elementwise kernel, the known-size "
                         "reference that hardware-counter runs are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2601_04707_amd import mqg, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda"
    w = synth.WORKLOADS[args.workload]
    if args.scale != 1.0:
        w = synth.scaled(w, args.scale)
    cache_pct = args.cache_pct if args.cache_pct is not None else w.cache_pct
    K, W = args.steps, args.warmup
    nfl = max(1, args.in_flight)
    L = len(w.fanouts)
    elt = 2 if w.feat_dtype == torch.float16 else 4
    row_bytes = w.dim * elt

    # ---------------------------------------------------------------- inputs (untimed)
    t0 = time.time()
    rp, ci = synth.build_graph(w, seed=0, device=dev)
    n = rp.numel() - 1
    # pinned host rows on 64-byte boundaries where that is cheap (synth.aligned_row_stride; measured on
    # "medium": 2.41 instead of 2.54 ms/step)
    feats = synth.pinned_features(n, w.dim, dtype=w.feat_dtype, seed=1, device=dev)
    torch.cuda.synchronize()
    g = mqg.Graph(rp, ci)
    batches = synth.seed_batches(n, w.batch, K + W, seed=2, train_fraction=w.train_fraction)
    seeds_dev = [b.to(g.idx_dtype).to(dev) for b in batches]
    gen_s = time.time() - t0

    # the same alignment rule for the rows in HBM (cache, gathered rows, layer outputs): measured on
    # "medium" 46.7 instead of 48.9 us for the hit gather, 101 instead of 103 us for the aggregation
    pad_dim = synth.aligned_row_stride(w.dim, w.feat_dtype)
    if args.device_row_multiple:
        m = args.device_row_multiple
        pad_dim = (row_bytes + m - 1) // m * m // elt
    ctxs = [mqg.Context(g, w.batch, w.fanouts) for _ in range(nfl)]
    blks = [mqg.Blocks(g, w.batch, w.fanouts) for _ in range(nfl)]
    streams = [torch.cuda.Stream() for _ in range(nfl)] if (nfl > 1 or args.graph) else [torch.cuda.current_stream()]
    if cache_pct is None:
        cache = mqg.Cache(g, feats.to(dev), None)
        num_cached = 0
    else:
        num_cached = n * cache_pct // 100
        cache = mqg.Cache(g, feats, num_cached, cache_stride=pad_dim)
        train_dev = None
        if args.cache_policy in ("walk", "walk-sampled"):
            # the training set: every node the seed batches are drawn from
            gen = torch.Generator()
            gen.manual_seed(2)
            perm = torch.randperm(n, generator=gen)
            train = perm if w.train_fraction is None else perm[: max(w.batch, int(n * w.train_fraction))]
            train_dev = train.to(g.idx_dtype).to(dev)
            torch.cuda.synchronize()
        t0 = time.time()
        if args.cache_policy == "top":
            mqg.mqg_build_cache(ctxs[0], g, cache)
        elif args.cache_policy == "sampled":
            mqg.mqg_build_cache_ex(ctxs[0], g, cache, mqg.MQG_CACHE_DEGREE_SAMPLED, seed=5)
        else:
            policy = mqg.MQG_CACHE_RANDOM_WALK if args.cache_policy == "walk" else mqg.MQG_CACHE_RANDOM_WALK_SAMPLED
            mqg.mqg_build_cache_ex(ctxs[0], g, cache, policy, seed=5, train_ids=train_dev,
                                   step_fanouts=list(reversed(w.fanouts)))
        torch.cuda.synchronize()
    build_cache_ms = (time.time() - t0) * 1e3 if cache_pct is not None else 0.0
    if args.prioritise_cache:
        if cache_pct is None:
            print("bench.py: --prioritise-cache needs a cache", file=sys.stderr)
            return 2
        for c in ctxs:
            c.set_sampling_priority(cache)
        torch.cuda.synchronize()

    for c in ctxs:
        if args.miss_inflight_kb is not None:
            c.set_option(mqg.MQG_OPT_MISS_INFLIGHT_BYTES, args.miss_inflight_kb * 1024)
        if args.heavy_degree is not None:
            c.set_option(mqg.MQG_OPT_HEAVY_DEGREE, args.heavy_degree)
        if args.dedup == "hash":
            c.set_option(mqg.MQG_OPT_DEDUP_HASH, 1)
    bounds = blks[0].bounds
    x0 = [torch.zeros((bounds[0][1], pad_dim), dtype=w.feat_dtype, device=dev)[:, :w.dim] for _ in range(nfl)]
    hs = [[torch.zeros((bounds[l][0], pad_dim), dtype=w.feat_dtype, device=dev)[:, :w.dim] for l in range(L)] for _ in range(nfl)]
    stats = [torch.zeros(2, dtype=torch.int64, device=dev) for _ in range(nfl)]
    sizes_log = torch.zeros((K + W, L, 4), dtype=torch.int64, device=dev)
    stats_log = torch.zeros((K + W, 2), dtype=torch.int64, device=dev)
    base_seed = 3

    def step(i: int):
        j = i % nfl
        s = streams[j]
        with torch.cuda.stream(s):
            mqg.mqg_sample_blocks(ctxs[j], g, seeds_dev[i], w.fanouts, base_seed + i, blks[j], stream=s)
            mqg.mqg_gather_features(ctxs[j], cache, blks[j].src_ids[0], blks[j].sizes[0, 1:2], x0[j], stats[j], stream=s)
            x = x0[j]
            for l in range(L):
                mqg.mqg_sage_mean_aggregate(ctxs[j], blks[j], l, x, hs[j][l], stream=s)
                x = hs[j][l]
            sizes_log[i].copy_(blks[j].sizes, non_blocking=True)
            stats_log[i].copy_(stats[j], non_blocking=True)

    timed_step = step
    if args.graph:
        # one recorded step per in-flight slot; what changes between replays lives in device buffers
        seed_buf = [torch.zeros(w.batch, dtype=g.idx_dtype, device=dev) for _ in range(nfl)]
        rng_buf = [torch.zeros(1, dtype=torch.int64, device=dev) for _ in range(nfl)]
        rng_vals = torch.arange(base_seed, base_seed + K + W, dtype=torch.int64, device=dev)

        def recorded(j):
            s = streams[j]
            mqg.mqg_sample_blocks_seed_dev(ctxs[j], g, seed_buf[j], w.fanouts, rng_buf[j], blks[j], stream=s)
            mqg.mqg_gather_features(ctxs[j], cache, blks[j].src_ids[0], blks[j].sizes[0, 1:2], x0[j], stats[j], stream=s)
            x = x0[j]
            for l in range(L):
                mqg.mqg_sage_mean_aggregate(ctxs[j], blks[j], l, x, hs[j][l], stream=s)
                x = hs[j][l]

        for i in range(nfl):                                    # eager once, then record
            step(i)
        torch.cuda.synchronize()
        graphs = []
        for j in range(nfl):
            seed_buf[j].copy_(seeds_dev[j])
            cg = torch.cuda.CUDAGraph()
            with torch.cuda.graph(cg, stream=streams[j]):
                recorded(j)
            graphs.append(cg)
        torch.cuda.synchronize()

        def timed_step(i: int):
            j = i % nfl
            with torch.cuda.stream(streams[j]):
                seed_buf[j].copy_(seeds_dev[i], non_blocking=True)
                rng_buf[j].copy_(rng_vals[i:i + 1], non_blocking=True)
                graphs[j].replay()
                sizes_log[i].copy_(blks[j].sizes, non_blocking=True)
                stats_log[i].copy_(stats[j], non_blocking=True)

    # ---------------------------------------------------------------- timed region
    for i in range(W):
        timed_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(W, W + K):
        timed_step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    sizes_host = sizes_log[W:].cpu().numpy()
    stats_host = stats_log[W:].cpu().numpy()
    edges = int(sizes_host[:, :, 2].sum())
    rows = int(sizes_host[:, 0, 1].sum())
    hits, misses = int(stats_host[:, 0].sum()), int(stats_host[:, 1].sum())
    ms_per_step = elapsed / K * 1e3
    edges_per_s = edges / elapsed
    gather_bytes = rows * row_bytes

    # ---------------------------------------------------------------- per-kernel durations
    # HIP events on the launch stream around every kernel (MQG_OPT_PROFILE), one mini-batch at a
    # time so that a kernel's duration is its own and not that of whatever overlaps it.
    for c in ctxs:
        c.set_option(mqg.MQG_OPT_PROFILE, 1)
    keys_eval, keys_batches = 0, 0
    for i in range(W, W + K):
        step(i)
        torch.cuda.synchronize()
        if keys_batches < 8:
            # random keys the sampler must evaluate: the whole adjacency row of every destination
            # whose degree exceeds the fanout (a row that fits is copied without any key)
            j = i % nfl
            for l in range(L):
                nd = int(blks[j].sizes[l, 0])
                dst = blks[j].src_ids[l][:nd].to(torch.int64)
                deg = (rp[dst + 1] - rp[dst]).to(torch.int64)
                keys_eval += int(deg[deg > w.fanouts[l]].sum())
            keys_batches += 1
    kernels = {}
    for c in ctxs:
        for name in c.kernel_names():
            ms, cnt = c.kernel_time(name)
            a = kernels.setdefault(name, [0.0, 0])
            a[0] += ms
            a[1] += cnt
        c.set_option(mqg.MQG_OPT_PROFILE, 0)
    kern = {k: {"launches": v[1], "avg_us": round(v[0] / max(v[1], 1) * 1e3, 3),
                "us_per_step": round(v[0] / K * 1e3, 3)} for k, v in sorted(kernels.items())}

    def pmc_traffic(kernel):
        """HBM bytes per launch from the committed rocprofv3 FETCH_SIZE/WRITE_SIZE summary, if it
        covers this workload (lines `traffic <workload> <kernel> <bytes>` in profiles/*.md)."""
        import glob
        for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
            for line in open(path):
                f = line.split()
                if len(f) == 4 and f[0] == "traffic" and f[1] == w.name and f[2] == kernel:
                    return int(f[3])
        return None

    def roof(name, bytes_per_launch, peak, traffic=None):
        if name not in kernels or kernels[name][1] == 0:
            return None
        avg_s = kernels[name][0] / kernels[name][1] * 1e-3
        ach = bytes_per_launch / avg_s / 1e9
        return {"kernel": name, "bound": "hbm", "achieved": round(ach, 1), "peak": peak, "unit": "GB/s",
                "frac": round(ach / peak, 4), "traffic": traffic,
                "avg_kernel_us": round(avg_s * 1e6, 2), "bytes_per_launch": int(bytes_per_launch)}

    if cache_pct is None:
        # direct gather: row read + row written + the id
        roofline = roof("k_gather_direct", rows / K * (2 * row_bytes + ci.element_size()), HBM_PEAK_GBPS,
                        pmc_traffic("k_gather_direct"))
        host_link = None
    else:
        # hit gather: row read from the HBM cache + row written + the 8-byte (row, slot) list entry
        roofline = roof("k_gather_hit", hits / K * (2 * row_bytes + 8), HBM_PEAK_GBPS, pmc_traffic("k_gather_hit"))
        host_link = roof("k_gather_miss", misses / K * row_bytes, HOST_LINK_PEAK_GBPS)
        if host_link:
            host_link["bound"] = "host-link"

    # the forward profile pass launches nothing else through the radix/scan kernels than the hash dedup
    dedup_kernels = ("k_bitmap_count", "k_bitmap_emit", "k_relabel", "k_reset_local", "k_zero_u64", "k_scan_tiles(radix)",
                     "k_scan_tiles(bitmap)", "k_scan_reduce", "k_scan_apply")
    dedup_us = sum(v["us_per_step"] for k, v in kern.items()
                   if k in dedup_kernels or k.startswith("k_hash_") or k.startswith("k_radix_"))
    sample_us = dedup_us + sum(v["us_per_step"] for k, v in kern.items()
                               if k in ("k_init_seeds", "k_row_info", "k_scan_tiles(rows)", "k_row_offsets", "k_sample",
                                        "k_sample_prio"))
    gather_us = sum(v["us_per_step"] for k, v in kern.items() if k.startswith("k_gather") or k in ("k_classify", "k_fill_u64", "k_direct_stats"))
    agg_us = kern.get("k_mean_aggregate", {}).get("us_per_step", 0.0)
    # ---------------------------------------------------------------- sampling against its own bounds
    # Integer ALU: one key costs 5 32-bit multiplies (quarter rate) and about 17 full-rate integer
    # operations = 37 lane-cycles; the chip has 256 CUs x 4 SIMDs x 16 lanes at 2.4 GHz.
    keys_per_step = keys_eval / max(keys_batches, 1)
    alu_peak_keys = 256 * 4 * 16 * 2.4e9 / 37.0
    k_sample_us = kern.get("k_sample_prio" if args.prioritise_cache else "k_sample", {}).get("us_per_step", 0.0)
    sampling = {
        "edges_per_s_sampling_alone": round(edges / K / max(sample_us, 1e-9) * 1e6, 1),
        "us_per_step": round(sample_us, 1), "kernel_launches_per_step": sum(
            v["launches"] for k, v in kern.items() if k in ("k_row_info", "k_scan_tiles(rows)", "k_scan_tiles(bitmap)", "k_row_offsets",
                                                            "k_sample", "k_sample_prio", "k_bitmap_count", "k_bitmap_emit", "k_relabel", "k_reset_local")) / K,
        "keys_evaluated_per_step": round(keys_per_step, 1),
        "k_sample": {"bound": "alu", "achieved": round(keys_per_step / max(k_sample_us, 1e-9) * 1e-3, 2),
                     "peak": round(alu_peak_keys / 1e9, 1), "unit": "Gkeys/s",
                     "frac": round(keys_per_step / max(k_sample_us, 1e-9) * 1e6 / alu_peak_keys, 4)},
        # 12 B of row information per destination plus, per sampled edge, the index read, the
        # neighbour written and read back, one local_of probe and the relabelled index written
        "hbm_frac_of_algorithmic_bytes": round(((edges / K) * (ci.element_size() + 16) + (sizes_host[:, :, 0].sum() / K) * 12)
                                               / max(sample_us, 1e-9) * 1e6 / (HBM_PEAK_GBPS * 1e9), 5),
    }

    # ---------------------------------------------------------------- the paper's queue-depth rule on these timings
    whole = lambda t: t._base if t._base is not None else t       # the padded allocation behind a column view
    per_batch_bytes = sum(t.numel() * t.element_size() for t in
                          [whole(x0[0])] + [whole(h) for h in hs[0]] + blks[0].src_ids + blks[0].indptr + blks[0].indices)
    try:
        q_rule, q_cap = mqg.mqg_queue_size(max((sample_us + gather_us) * 1e-3, 1e-6), max(agg_us * 1e-3, 1e-6),
                                           torch.cuda.get_device_properties(0).total_memory,
                                           torch.cuda.max_memory_allocated(), 10, per_batch_bytes)
    except mqg.MqgError:
        q_rule, q_cap = None, None

    # ---------------------------------------------------------------- backward of the aggregation chain
    # Not part of a step.  A pass of its own (so that it does not disturb the caches of the kernels
    # timed above): per mini-batch the forward path, then the gradient of the last block's output
    # pushed back through every block to the gathered rows, one mini-batch at a time.
    for c in ctxs:
        c.reset_profile()
        c.set_option(mqg.MQG_OPT_PROFILE, 1)
    gx = [torch.zeros((bounds[l][1], pad_dim), dtype=w.feat_dtype, device=dev)[:, :w.dim] for l in range(L)]
    g_top = torch.randn((bounds[L - 1][0], pad_dim), device=dev).to(w.feat_dtype)[:, :w.dim]
    # the same pass also runs the weighted (graph-convolution, paper Eq. 1-3) variant of the aggregation
    # chain on the same blocks: weights of every block, then the weighted sums
    ew = [torch.zeros(bounds[l][2], dtype=torch.float32, device=dev) for l in range(L)]
    sw = [torch.zeros(bounds[l][0], dtype=torch.float32, device=dev) for l in range(L)]
    KB = min(K, 50)
    for i in range(W, W + KB):
        step(i)
        j = i % nfl
        with torch.cuda.stream(streams[j]):
            gcur = g_top
            for l in range(L - 1, -1, -1):
                mqg.mqg_sage_mean_aggregate_backward(ctxs[j], blks[j], l, gcur, gx[l], stream=streams[j])
                gcur = gx[l]
            x = x0[j]
            for l in range(L):
                mqg.mqg_gcn_edge_weights(ctxs[j], g, blks[j], l, ew[l], sw[l], stream=streams[j])
                mqg.mqg_weighted_aggregate(ctxs[j], blks[j], l, ew[l], sw[l], x, hs[j][l], stream=streams[j])
                x = hs[j][l]
        torch.cuda.synchronize()
    wk = {}
    for c in ctxs:
        for name in ("k_gcn_edge_weights", "k_weighted_aggregate"):
            ms, cnt = c.kernel_time(name)
            a = wk.setdefault(name, [0.0, 0])
            a[0] += ms
            a[1] += cnt
    wagg_us = wk["k_weighted_aggregate"][0] / KB * 1e3
    wgt_us = wk["k_gcn_edge_weights"][0] / KB * 1e3
    bwd_names = ("k_edge_dst_rows", "k_radix_hist", "k_scan_reduce", "k_scan_tiles(radix)", "k_scan_apply",
                 "k_radix_scatter", "k_col_ptr", "k_mean_aggregate_backward")
    bk = {}
    for c in ctxs:
        for name in bwd_names:
            ms, cnt = c.kernel_time(name)
            a = bk.setdefault(name, [0.0, 0])
            a[0] += ms
            a[1] += cnt
        c.set_option(mqg.MQG_OPT_PROFILE, 0)
    bwd_us = sum(v[0] for v in bk.values()) / KB * 1e3
    bwd_kernel_us = bk["k_mean_aggregate_backward"][0] / KB * 1e3
    # reduction kernel: every edge reads one gradient row, every source row of every block is written once
    bwd_bytes = (edges + int(sizes_host[:, :, 1].sum())) / K * row_bytes

    # ---------------------------------------------------------------- layer-wise (LADIES) mini-batches
    # Not part of a step either: the paper's layer-wise setting (512 nodes per layer) on the same
    # seeds - sampling, gather of the outermost layer's rows, weighted sums - one batch at a time.
    lw_sizes = [512] * L
    lw_blocks = mqg.LayerwiseBlocks(g, w.batch, lw_sizes, nnz_per_row=512)
    lw_x0 = torch.zeros((lw_blocks.bounds[0][1], pad_dim), dtype=w.feat_dtype, device=dev)[:, :w.dim]
    lw_h = [torch.zeros((lw_blocks.bounds[l][0], pad_dim), dtype=w.feat_dtype, device=dev)[:, :w.dim] for l in range(L)]
    lw_stats = torch.zeros(2, dtype=torch.int64, device=dev)
    c0 = ctxs[0]

    def lw_step(i, method=0):
        mqg.mqg_sample_layerwise(c0, g, seeds_dev[i], lw_sizes, base_seed + i, lw_blocks, method=method)
        mqg.mqg_gather_features(c0, cache, lw_blocks.src_ids[0], lw_blocks.sizes[0, 1:2], lw_x0, lw_stats)
        x = lw_x0
        for l in range(L):
            mqg.mqg_weighted_aggregate(c0, lw_blocks, l, lw_blocks.edge_w[l], None, x, lw_h[l])
            x = lw_h[l]

    lw_step(W)                                                  # allocates the sampler's scratch
    torch.cuda.synchronize()
    KL = min(K, 30)
    t0 = time.perf_counter()
    for i in range(W, W + KL):
        lw_step(i)
    torch.cuda.synchronize()
    lw_ms = (time.perf_counter() - t0) / KL * 1e3
    lw_edges = int(lw_blocks.sizes[:, 2].sum())
    # the variants the paper's tables list (FastGCN's batch-independent masses, flat probabilities, debiasing)
    lw_variants = {}
    for name, method in (("fastgcn", mqg.MQG_LAYERWISE_FASTGCN),
                         ("ladies+f+d", mqg.MQG_LAYERWISE_FLAT | mqg.MQG_LAYERWISE_DEBIAS),
                         ("fastgcn+f+d", mqg.MQG_LAYERWISE_FASTGCN | mqg.MQG_LAYERWISE_FLAT | mqg.MQG_LAYERWISE_DEBIAS)):
        lw_step(W, method)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(W, W + KL):
            lw_step(i, method)
        torch.cuda.synchronize()
        lw_variants[name] = round((time.perf_counter() - t0) / KL * 1e3, 3)
    c0.reset_profile()
    c0.set_option(mqg.MQG_OPT_PROFILE, 1)
    for i in range(W, W + KL):
        lw_step(i)
        torch.cuda.synchronize()
    lw_kern = {}
    for name in c0.kernel_names():
        ms, cnt = c0.kernel_time(name)
        if cnt:
            lw_kern[name] = round(ms / KL * 1e3, 1)
    c0.set_option(mqg.MQG_OPT_PROFILE, 0)
    lw_sample_us = sum(v for k, v in lw_kern.items() if k.startswith("k_lw_") or k.startswith("k_radix") or k.startswith("k_scan"))

    # ---------------------------------------------------------------- CPU baseline: the oracle, one thread
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        rp_np, ci_np = rp.cpu().numpy().astype(np.int64), ci.cpu().numpy().astype(np.int64)
        feats_np = feats.numpy()
        ocache = oracle.build_cache(rp_np, num_cached, feats_np) if cache_pct is not None else None
        nb = args.cpu_batches
        t_cpu, e_cpu, done = 0.0, 0, 0
        budget_s = 20.0
        for i in range(W, W + K):
            t1 = time.perf_counter()
            ob = oracle.sample_blocks(rp_np, ci_np, batches[i].numpy(), w.fanouts, base_seed + i)
            x, _, _ = oracle.gather(ob[0].src_ids, feats_np, ocache)
            for l in range(L):
                x = oracle.mean_aggregate(ob[l].indptr, ob[l].indices, x)
            t_cpu += time.perf_counter() - t1
            e_cpu += sum(b.nnz for b in ob)
            done += 1
            if i == W:   # the first oracle batch doubles as an end-to-end check of the timed GPU path
                assert [b.nnz for b in ob] == sizes_host[0, :, 2].tolist(), "GPU and oracle disagree on batch sizes"
            if (nb is not None and done >= nb) or (nb is None and t_cpu > budget_s):
                break
        cpu = {"value": round(e_cpu / t_cpu, 1), "unit": "sampled edges/s", "cores": 1, "kind": "oracle",
               "sample": f"first {done} of the {K} timed mini-batches, whole path (sample+gather+aggregate), "
                         f"{t_cpu:.1f} s; host has {os.cpu_count()} logical cores"}

    # ---------------------------------------------------------------- what plain copies reach on this machine (context)
    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3
    ca = torch.ones(1 << 27, dtype=torch.float32, device=dev)          # 512 MiB
    cb = torch.empty_like(ca)
    t_copy = timed(lambda: torch.mul(ca, 2.0, out=cb))
    hrows = max(1, min(n, (1 << 29) // (feats.stride(0) * feats.element_size())))
    hsrc = torch.as_strided(feats, (hrows * feats.stride(0),), (1,))       # whole rows including any padding
    nb = hsrc.numel() * feats.element_size()
    hdst = torch.empty_like(hsrc, device=dev)
    t_h2d = timed(lambda: hdst.copy_(hsrc, non_blocking=True))
    measured = {"hbm_read_plus_write_GBps": round(2 * ca.numel() * 4 / t_copy / 1e9, 1),
                "pinned_host_to_device_GBps": round(nb / t_h2d / 1e9, 1)}
    del ca, cb, hdst

    if args.pmc_copy:
        a = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        torch.mul(a, 2.0, out=b)
        torch.cuda.synchronize()

    out = {
        "metric": "sampled edges/sec + feature-gather GB/s (% of HBM peak) per mini-batch",
        "value": round(edges_per_s, 1),
        "unit": "sampled edges/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64+f32" if elt == 4 else "int64+f16",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: Chung-Lu power-law graph, {n} nodes, {ci.numel()} directed edges, "
                               f"{w.dim}-dim {'fp32' if elt == 4 else 'fp16'} features, fanouts {w.fanouts}, "
                               f"{w.batch} seeds/batch, HBM cache {cache_pct if cache_pct is not None else 'all'} % of nodes ({args.cache_policy}), "
                               f"rest in pinned host memory ({feats.stride(0) * elt}-byte rows)",
                   "in_flight": nfl, "global_batch": w.batch, "dedup": args.dedup,
                   "sampling": "cached neighbours first" if args.prioritise_cache else "uniform",
                   "launch": "one recorded HIP graph per in-flight slot" if args.graph else "eager"},
        "gather_GBps": round(gather_bytes / elapsed / 1e9, 2),
        "gather_kernel_GBps": round(gather_bytes / K / max(gather_us, 1e-9) * 1e-3, 2),
        "edges_per_step": round(edges / K, 1), "rows_per_step": round(rows / K, 1),
        "cache_hit_rate": round(hits / max(1, hits + misses), 4),
        "stage_us_per_step": {"sample": round(sample_us, 1), "gather": round(gather_us, 1), "aggregate": round(agg_us, 1),
                              "dedup_relabel_part_of_sample": round(dedup_us, 1)},
        "backward_aggregation": {"us_per_step": round(bwd_us, 1), "reduction_kernel_us_per_step": round(bwd_kernel_us, 1),
                                 "reduction_kernel_GBps": round(bwd_bytes / max(bwd_kernel_us, 1e-9) * 1e-3, 1),
                                 "note": "all blocks of a mini-batch, one at a time; not part of a step"},
        "gcn_weighted_aggregation": {"weights_kernel_us_per_step": round(wgt_us, 1), "sum_kernel_us_per_step": round(wagg_us, 1),
                                     "mean_aggregate_us_per_step": round(agg_us, 1),
                                     "note": "Eq. 1-3 estimator on the same blocks (weights of every block, then weighted "
                                             "sums with the diagonal term); not part of a step"},
        "layerwise_sampling": {"layer_sizes": lw_sizes, "ms_per_batch": round(lw_ms, 3),
                               "sampling_kernels_us_per_batch": round(lw_sample_us, 1),
                               "edges_last_batch": lw_edges, "kernel_us_per_batch": lw_kern,
                               "variants_ms_per_batch": lw_variants,
                               "note": "LADIES (Eq. 6-9) on the same seeds: sample, gather, weighted sums, one "
                                       "mini-batch at a time on one stream; not part of a step"},
        "sampling": sampling,
        "paper_queue_rule": {"queue_size": q_rule, "memory_cap": q_cap, "bytes_per_queued_batch": per_batch_bytes,
                             "note": "Eq. 22-23 on mean prepare (sample+gather) / consume (aggregate) times of this run; "
                                     "the depth actually used is config.in_flight: the path is bound by the host link, "
                                     "which three mini-batches already keep busy"},
        "roofline": roofline,
        "roofline_host_link": host_link,
        "measured_plain_copies": measured,
        "cpu_baseline": cpu,
        "kernels": kern,
        "build_cache_ms": round(build_cache_ms, 2),
        "input_generation_s": round(gen_s, 1),
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
