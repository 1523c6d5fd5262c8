#!/usr/bin/env python3
"""Benchmark of the dual-cache GNN inference hot path on one MI355X.

A step is one pass of the per-batch path (cache-aware k-hop sampling -> cache-aware feature
gather -> GraphSAGE-mean forward) over one mini-batch of the workload; the one-off part of the
path (pre-sampling counts, Eq. (1) split, dual-cache fill) runs before the timed region and is
reported separately.  Inputs are seeded synthetic R-MAT graphs / Gaussian features / Glorot
weights with the shapes of the paper's datasets, resident in pinned host memory (graph,
features) and HBM (caches, seeds, weights) when the timed region starts.

Prints ONE JSON line.  `value` is sampled edges per second over whole steps; the gather
bandwidth, hit rates and per-kernel times ride along, plus
  roofline     - the dominant kernel against MI355X's published peak, timed with HIP events
                 inside the timed region;
  cpu_baseline - the CPU oracle timed on this machine's host cores on a bounded sample.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
FP32_MFMA_PEAK_TFLOPS = 157.3
PIN_LIMIT_BYTES = 60 * 10**9     # the GPU machines refuse page-locked allocations beyond 64 GiB in total


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=54)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="medium", choices=["tiny", "medium", "large", "huge", "skewed", "yelp", "amazon"])
    ap.add_argument("--placement", default="auto", choices=["auto", "host", "indices-hbm", "features-hbm"],
                    help="where the graph and the features live: 'host' = all in pinned host memory; 'indices-hbm' = "
                         "features and list bounds pinned, neighbour ids in HBM; 'features-hbm' = graph pinned, features "
                         "in HBM; 'auto' = 'host' when graph + features fit the pinned-memory limit, else 'indices-hbm'")
    ap.add_argument("--no-cache", action="store_true", help="run the miss path only (no dual cache)")
    ap.add_argument("--feat-policy", type=int, default=0)
    ap.add_argument("--budget", type=float, default=None, help="cache budget in bytes (default: the workload's)")
    ap.add_argument("--n-presample", type=int, default=None, help="pre-sampled batches (default: the workload's 8)")
    ap.add_argument("--single-cache", action="store_true",
                    help="the paper's single-cache comparison: the whole budget goes to features, no adjacency cache")
    ap.add_argument("--adj-elements", action="store_true",
                    help="element-granular adjacency cache (Algorithm 1 as printed): lists reordered by element count, "
                         "last node cached in part; pre-sampling then also counts per element")
    ap.add_argument("--model", default="sage-mean", choices=["sage-mean", "sage-sum", "gcn-avg"],
                    help="GNN of the forward pass (Table III); the headline configuration is sage-mean")
    ap.add_argument("--linear-kernel", type=int, default=0, choices=[0, 1, 2, 3],
                    help="dense-layer kernel of the timed region: 0 by shape (default), 1 register-staged tile kernel, "
                         "2 wide kernel, 3 by shape without the wide kernel")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-batches", type=int, default=8, help="batches the CPU oracle is timed on")
    ap.add_argument("--streams", type=int, default=1,
                    help="HIP streams of the timed region; each runs whole steps on its share of the batches. The "
                         "default 1 keeps every kernel alone on the chip so that the per-kernel roofline is clean")
    ap.add_argument("--extra-streams", type=int, default=4,
                    help="after the timed region, time the same K steps once more on this many streams and report "
                         "it under extras.multi_stream (0 = skip)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the timed region run one device-to-device copy of 1 GiB (a kernel of known "
                         "traffic for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--time-all-kernels", action="store_true",
                    help="bracket every kernel class with events (perturbs the step time slightly)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2503_01281_amd as dci
    import synth

    w = synth.WORKLOADS[args.workload]
    if args.budget is not None:
        w = w.scaled(w.name, budget_bytes=int(args.budget))
    if args.n_presample is not None:
        w = w.scaled(w.name, n_presample=args.n_presample)
    torch.cuda.set_device(0)
    t0 = time.time()
    # Placement.  The graph and the feature matrix belong in pinned host memory (zero-copy misses over the host
    # link).  A GPU machine pins at most 64 GiB, less than the two largest workloads need (70.7 / 81.5 GB), so for
    # those the feature matrix and the list-bound array stay pinned and the neighbour-id array - which the
    # adjacency cache covers in full or nearly so at their budgets - is placed in HBM, standing in for the host tier.
    place = args.placement
    if place == "auto":
        place = "host" if w.adj_bytes + w.feat_bytes <= PIN_LIMIT_BYTES else "indices-hbm"
    indptr = dci.pinned_empty(w.num_nodes + 1, torch.int64)
    if place in ("host", "features-hbm"):
        indices = dci.pinned_empty(w.num_edges, torch.int64)
        indices_host = indices
    else:
        indices_host = torch.empty(w.num_edges, dtype=torch.int64)
    synth.rmat_csr(w.num_nodes, w.num_edges, w.rmat, w.graph_seed, indptr_ptr=indptr.data_ptr(),
                   indices_ptr=indices_host.data_ptr())
    if place == "indices-hbm":
        indices = torch.empty(w.num_edges, dtype=torch.int64, device="cuda")
        for lo_ in range(0, w.num_edges, 1 << 27):
            indices[lo_:lo_ + (1 << 27)].copy_(indices_host[lo_:lo_ + (1 << 27)])
    feat_in_hbm = place == "features-hbm"
    if feat_in_hbm:
        feat_host = torch.from_numpy(synth.features(w.num_nodes, w.feat_dim, w.feature_seed))
        feat = torch.empty(w.num_nodes, w.feat_dim, dtype=torch.float32, device="cuda")
        rows_step = max(1, (1 << 28) // w.feat_dim)
        for lo_ in range(0, w.num_nodes, rows_step):
            feat[lo_:lo_ + rows_step].copy_(feat_host[lo_:lo_ + rows_step])
    else:
        feat = dci.pinned_empty(w.num_nodes * w.feat_dim, torch.float32).view(w.num_nodes, w.feat_dim)
        synth.features(w.num_nodes, w.feat_dim, w.feature_seed, ptr=feat.data_ptr())
        feat_host = feat
    seeds_h = synth.seeds(w.num_nodes, w.num_seeds, w.seed_seed)
    ws_h, wn_h, b_h = synth.sage_weights(w.dims, w.weight_seed)
    log(f"[bench] inputs for '{w.name}' generated in {time.time() - t0:.1f}s "
        f"(N={w.num_nodes} E={w.num_edges} F={w.feat_dim})")

    ctx = dci.Context(0)
    g = dci.Graph(indptr, indices, feat)
    seeds = torch.from_numpy(seeds_h).cuda()
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    ws, wn, bs = [dev(a) for a in ws_h], [dev(a) for a in wn_h], [dev(a) for a in b_h]
    blk = dci.Blocks(ctx, w.num_nodes, w.batch_size, w.fanouts)
    x = torch.empty(blk.cap_nodes[-1], w.feat_dim, dtype=torch.float32, device="cuda")
    logits = torch.empty(w.batch_size, w.classes, dtype=torch.float32, device="cuda")

    # ---- one-off part: pre-sampling counts (timed per stage for Eq. (1)) and the dual-cache fill
    cache = None
    pre = {}
    if not args.no_cache:
        fc = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
        ac = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
        stats = torch.zeros(dci.STATS_WORDS, dtype=torch.int64, device="cuda")
        ec = torch.zeros(w.num_edges, dtype=torch.int32, device="cuda") if args.adj_elements else None
        fill_flags = args.feat_policy | (dci.DCI_FILL_ADJ_ELEMENTS if args.adj_elements else 0)
        ctx.sync()
        t0 = time.time()
        dci.dci_presample_count(ctx, g, None, seeds, w.batch_size, 0, w.n_presample, w.presample_first_batch,
                                w.fanouts, w.rng_seed, fc, ac, ec, feat_scratch=x, stats=stats)
        ctx.sync()
        t1 = time.time()
        st = stats.cpu().numpy()
        ts, tf = int(st[dci.STAT["t_sample_ns"]]), int(st[dci.STAT["t_feature_ns"]])
        if args.single_cache:
            cache = dci.dci_fill_caches(ctx, g, fc, ac, w.budget_bytes, 0, 1, fill_flags | dci.DCI_FILL_STRICT_SPLIT,
                                        edge_count=ec)
        else:
            cache = dci.dci_fill_caches(ctx, g, fc, ac, w.budget_bytes, ts, tf, fill_flags, edge_count=ec)
        del ec
        t2 = time.time()
        pre = dict(presample_s=round(t1 - t0, 4), fill_s=round(t2 - t1, 4), t_sample_ns=ts, t_feature_ns=tf,
                   cap_adj_bytes=int(cache.cap_adj_bytes), cap_feat_bytes=int(cache.cap_feat_bytes),
                   adj_nodes=int(cache.adj_nodes), adj_edges=int(cache.adj_edges), feat_rows=int(cache.feat_rows),
                   adj_elements=bool(args.adj_elements), adj_partial_node=int(cache.adj_partial_node))
        log(f"[bench] preprocess: {pre}")

    nb = w.num_batches

    # Batches are independent, so S streams each run whole steps (sample -> gather -> forward, own
    # context, workspace and buffers) on batches b = s (mod S): the short latency-bound sampling
    # kernels, the bandwidth-bound gather / mean and the MFMA-bound dense layers of different batches
    # then share the chip.  All streams have the default priority.
    n_streams = max(1, args.streams, args.extra_streams)  # buffers for the larger of the two regions
    main = torch.cuda.current_stream()
    streams = [main] + [torch.cuda.Stream() for _ in range(n_streams - 1)]
    ctxs = [ctx] + [dci.Context(0, stream=st_) for st_ in streams[1:]]
    blks = [blk] + [dci.Blocks(ctx, w.num_nodes, w.batch_size, w.fanouts) for _ in range(n_streams - 1)]
    xs = [x] + [torch.empty_like(x) for _ in range(n_streams - 1)]
    outs = [logits] + [torch.empty_like(logits) for _ in range(n_streams - 1)]
    ws_need = ctx.lib.dci_sample_workspace_bytes(w.num_nodes, w.batch_size, (C.c_int32 * w.n_hops)(*w.fanouts), w.n_hops)
    sg_need = ctx.lib.dci_sage_workspace_bytes((C.c_int64 * 8)(*(blk.cap_nodes[:w.n_hops] + [0] * (8 - w.n_hops))),
                                               w.n_hops, (C.c_int32 * (w.n_hops + 1))(*w.dims))
    for c_ in ctxs:
        c_.ensure_workspace(max(ws_need, sg_need, 1 << 20))
    torch.cuda.synchronize()

    model = {"sage-mean": 0, "sage-sum": 1, "gcn-avg": 2}[args.model]
    k_ops = 1 if model == 2 else 2      # operands of the dense layer's contraction (GCN has one weight matrix)

    def step(b: int, k: int, stats_t):
        lo = (b % nb) * w.batch_size
        c_, bk = ctxs[k], blks[k]
        dci.dci_sample_khop(c_, g, cache, seeds[lo:lo + w.batch_size], b % nb, w.fanouts, w.rng_seed, bk, stats_t)
        dci.dci_gather_features(c_, g, cache, bk.nodes, bk.cap_nodes[-1], xs[k], n_dev=bk.n_input_dev(), stats=stats_t)
        if model == 0:
            dci.dci_sage_forward(c_, bk, xs[k], ws, wn, bs, outs[k])
        else:
            dci.dci_gnn_forward(c_, bk, xs[k], model, ws, wn, bs, outs[k])

    def run_steps(first: int, count: int, stats_list, use_streams: int):
        """Exactly `count` whole steps (batches first .. first+count-1); nothing is in flight before or after."""
        for st_ in streams[1:use_streams]:
            st_.wait_stream(main)
        for b in range(first, first + count):
            k = (b - first) % use_streams
            with torch.cuda.stream(streams[k]):
                step(b, k, None if stats_list is None else stats_list[k])
        for st_ in streams[1:use_streams]:
            main.wait_stream(st_)

    for c_ in ctxs:
        c_.set_option(dci.DCI_OPT_LINEAR_KERNEL, args.linear_kernel)
    run_steps(0, args.warmup, None, max(1, args.streams))
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps; the dominant kernel class is bracketed by events
    dominant = "linear_in"
    for c_ in ctxs:
        c_.timing_enable(dci.KERNEL_CLASSES if args.time_all_kernels else [dominant, "gather"])
    stats_list = [torch.zeros(dci.STATS_WORDS, dtype=torch.int64, device="cuda") for _ in range(n_streams)]
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    run_steps(0, args.steps, stats_list, max(1, args.streams))
    ev[1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall_s = t1 - t0
    timing = {k: (0.0, 0) for k in dci.KERNEL_CLASSES}
    for c_ in ctxs:
        for k, v in c_.timing_read().items():
            timing[k] = (timing[k][0] + v[0], timing[k][1] + v[1])
        c_.timing_enable([])
    stats = sum(stats_list[1:], stats_list[0])
    st = {k: int(v) for k, v in zip(dci.STAT.keys(), stats.cpu().numpy()[:len(dci.STAT)])}
    multi = None
    if args.extra_streams > 1:
        # with several batches in flight the statically partitioned wide dense-layer kernel (one workgroup per
        # compute unit) loses to the tile kernel, whose many small workgroups fill whatever the other streams leave
        for c_ in ctxs:
            c_.set_option(dci.DCI_OPT_LINEAR_KERNEL, 1)
        run_steps(0, min(args.steps, 2 * args.extra_streams), None, args.extra_streams)
        torch.cuda.synchronize()
        tm0 = time.perf_counter()
        run_steps(0, args.steps, None, args.extra_streams)
        torch.cuda.synchronize()
        tm = time.perf_counter() - tm0
        multi = {"streams": args.extra_streams, "linear_kernel": "tile", "ms_per_step": round(tm * 1e3 / args.steps, 4)}
        for c_ in ctxs:
            c_.set_option(dci.DCI_OPT_LINEAR_KERNEL, args.linear_kernel)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # host-link reference: one pinned-host -> HBM copy of the first GiB (or all) of the edge array
    link_src = indptr if not indices.is_pinned() else indices
    n_link = min(link_src.numel(), 1 << 27)
    link_dst = torch.empty(n_link, dtype=torch.int64, device="cuda")
    link_ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    link_dst.copy_(link_src[:n_link], non_blocking=True)
    torch.cuda.synchronize()
    link_ev[0].record()
    link_dst.copy_(link_src[:n_link], non_blocking=True)
    link_ev[1].record()
    torch.cuda.synchronize()
    host_link_gbps = n_link * 8 / (link_ev[0].elapsed_time(link_ev[1]) * 1e-3) / 1e9
    del link_dst

    edges = st["edges_sampled"]
    rows = st["feat_hits"] + st["feat_misses"]
    gather_bytes = rows * w.feat_dim * 4
    gather_ms, gather_n = timing["gather"]
    value = edges / wall_s
    if multi is not None:
        multi["value"] = round(edges / (multi["ms_per_step"] * 1e-3 * args.steps), 1)  # same K batches, same edges

    # ---- roofline of the dominant kernel: the first dense layer (fp32 MFMA, K = 2 * feat_dim).
    # Flops per launch are 2 * n_nodes[L-1] * (2 * dims[0]) * dims[1]; the row counts of the timed
    # batches are re-derived by sampling them again outside the timed region (sampling is a pure
    # function of the batch), the duration is the event time of the same launches.
    lin_ms, lin_n = timing[dominant]
    flops_in = flops_all = 0.0
    for b in range(args.steps):
        lo = (b % nb) * w.batch_size
        dci.dci_sample_khop(ctx, g, cache, seeds[lo:lo + w.batch_size], b % nb, w.fanouts, w.rng_seed, blk, None)
        ctx.sync()
        nn = blk.n_nodes()
        for l in range(w.n_hops):
            fl = 2.0 * nn[w.n_hops - 1 - l] * (k_ops * w.dims[l]) * w.dims[l + 1]
            flops_all += fl
            if l == 0:
                flops_in += fl
    lin_tflops = flops_in / (lin_ms * 1e-3) / 1e12 if lin_ms > 0 else 0.0
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath) and model == 0:   # the stored counters are of the GraphSAGE-mean launch
        try:
            traffic = json.load(open(tpath)).get(f"{dominant}:{w.name}")
        except Exception:
            traffic = None
    if args.linear_kernel in (0, 2) and w.dims[1] % 128 == 0 and w.dims[0] % 2 == 0 and (w.dims[0] >= 192 or args.linear_kernel == 2):
        lin_kernel = "k_sage_linear_wide"
    elif (args.linear_kernel in (0, 3) and w.dims[1] % 64 == 0 and w.dims[0] % 2 == 0
          and ((blk.cap_nodes[w.n_hops - 1] + 63) // 64 + 7) // 8 * 8 * (w.dims[1] // 64) > 128):   # else the split path
        lin_kernel = "k_sage_linear_dma"
    else:
        lin_kernel = "k_sage_linear"
    roofline = {"kernel": lin_kernel + " (first layer)", "bound": "mfma", "achieved": round(lin_tflops, 3),
                "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(lin_tflops / FP32_MFMA_PEAK_TFLOPS, 4),
                "traffic": traffic, "launches": lin_n, "avg_launch_ms": round(lin_ms / max(lin_n, 1), 4),
                "flops_per_launch": round(flops_in / max(lin_n, 1), 1)}
    gather_gbps = gather_bytes * 2 / (gather_ms * 1e-3) / 1e9 if gather_ms > 0 else 0.0
    gather_roof = {"kernel": "k_gather", "bound": "hbm", "achieved": round(gather_gbps, 1), "peak": HBM_PEAK_GBPS,
                   "unit": "GB/s", "frac": round(gather_gbps / HBM_PEAK_GBPS, 4),
                   "avg_launch_ms": round(gather_ms / max(gather_n, 1), 4),
                   "bytes_per_launch": round((gather_bytes * 2 + rows * 12) / max(gather_n, 1), 1)}

    # ---- CPU oracle on this machine's host cores, bounded sample: the first batch of the workload
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        ip, ix, ft = indptr.numpy(), indices_host.numpy(), feat_host.numpy()
        n_cpu = max(1, min(args.cpu_batches, nb))
        t_s = t_g = t_f = 0.0
        e_cpu = rows_cpu = 0
        for b in range(n_cpu):
            lo = b * w.batch_size
            c0 = time.perf_counter()
            ob_b = oracle.sample_khop(ip, ix, seeds_h[lo:lo + w.batch_size], b, w.fanouts, w.rng_seed)
            c1 = time.perf_counter()
            ox_b = oracle.gather(ft, ob_b.nodes)
            c2 = time.perf_counter()
            ol_b = oracle.gnn_forward(model, ob_b, ox_b, ws_h, wn_h, b_h)
            c3 = time.perf_counter()
            t_s += c1 - c0; t_g += c2 - c1; t_f += c3 - c2
            e_cpu += int(ob_b.n_edges.sum()); rows_cpu += len(ob_b.nodes)
            if b == 0:
                ob, ox, ol = ob_b, ox_b, ol_b
        cpu = {"value": round(e_cpu / (t_s + t_g + t_f), 1), "unit": "edges/s", "cores": 1, "kind": "oracle",
               "sample": f"batches 0..{n_cpu - 1} of '{w.name}' ({e_cpu} edges, {rows_cpu} input rows): "
                         f"sample {t_s:.2f}s, gather {t_g:.2f}s, forward {t_f:.2f}s",
               "sample_edges_per_s": round(e_cpu / t_s, 1),
               "gather_GBps": round(rows_cpu * w.feat_dim * 4 / t_g / 1e9, 3)}
        # the same batch from the GPU, as a last parity check on the benchmarked configuration
        dci.dci_sample_khop(ctx, g, cache, seeds[:w.batch_size], 0, w.fanouts, w.rng_seed, blk, None)
        dci.dci_gather_features(ctx, g, cache, blk.nodes, blk.cap_nodes[-1], x, n_dev=blk.n_input_dev())
        dci.dci_gnn_forward(ctx, blk, x, model, ws, wn, bs, logits)
        ctx.sync()
        nn = blk.n_nodes()
        ok_nodes = nn == [int(v) for v in ob.n_nodes] and bool(np.array_equal(blk.nodes[:nn[-1]].cpu().numpy(), ob.nodes))
        ok_src = all(np.array_equal(blk.blk_src[h][:blk.n_edges()[h]].cpu().numpy(), ob.blk_src[h]) for h in range(w.n_hops))
        ok_x = x[:nn[-1]].cpu().numpy().tobytes() == ox.tobytes()
        err = float(np.abs(logits[:w.batch_size].cpu().numpy() - ol).max())
        tol = 1e-4 * max(1.0, float(np.abs(ol).max()))
        cpu["parity"] = {"blocks_bit_exact": bool(ok_nodes and ok_src), "features_bit_exact": bool(ok_x),
                         "max_logit_err": err, "logit_tol": tol, "ok": bool(ok_nodes and ok_src and ok_x and err <= tol)}

    adj_total = st["adj_edge_hits"] + st["adj_edge_misses"]
    out = {
        "metric": "sampled edges/s through sample+gather+forward (gathered feature GB/s, hit rates in extras)",
        "value": round(value, 1), "unit": "edges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_s * 1e3 / args.steps, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "nodes": w.num_nodes, "edges": w.num_edges, "feat_dim": w.feat_dim,
                   "fanouts_from_seeds": list(w.fanouts), "batch_size": w.batch_size, "sage_dims": list(w.dims), "gnn": args.model,
                   "budget_bytes": 0 if args.no_cache else w.budget_bytes, "feat_policy": args.feat_policy,
                   "n_presample": w.n_presample, "single_cache": bool(args.single_cache),
                   "adj_elements": bool(args.adj_elements),
                   "cache": not args.no_cache, "streams": max(1, args.streams),
                   "placement": place,
                   "features": "hbm" if feat_in_hbm else "pinned host",
                   "indices": "hbm" if place == "indices-hbm" else "pinned host", "indptr": "pinned host"},
        "extras": {
            "edges_per_step": round(edges / args.steps, 1), "input_nodes_per_step": round(rows / args.steps, 1),
            "gather_GBps_delivered": round(gather_bytes / (gather_ms * 1e-3) / 1e9, 1) if gather_ms > 0 else None,
            "adj_hit_rate_edges": round(st["adj_edge_hits"] / adj_total, 4) if adj_total else None,
            "adj_hit_rate_nodes": round(st["adj_node_hits"] / max(1, st["adj_node_hits"] + st["adj_node_misses"]), 4),
            "feat_hit_rate": round(st["feat_hits"] / rows, 4) if rows else None,
            "gpu_event_ms_per_step": round(ev[0].elapsed_time(ev[1]) / args.steps, 4),
            "kernel_ms_per_step": {k: round(v[0] / args.steps, 4) for k, v in timing.items() if v[1]},
            "preprocess": pre,
            # pre-sampling + fill + one pass over all of the workload's batches at the measured step time
            "end_to_end_s": (round(pre["presample_s"] + pre["fill_s"] + wall_s / args.steps * nb, 4) if pre else
                             round(wall_s / args.steps * nb, 4)),
            "gather_roofline": gather_roof, "multi_stream": multi,
            "host_link_pinned_copy_GBps": round(host_link_gbps, 1),
            "gather_frac_of_host_link": (round(gather_bytes / (gather_ms * 1e-3) / 1e9 / host_link_gbps, 3)
                                         if (gather_ms > 0 and st["feat_hits"] == 0) else None),
        },
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
