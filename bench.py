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


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=54)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="medium", choices=["tiny", "medium", "large"])
    ap.add_argument("--no-cache", action="store_true", help="run the miss path only (no dual cache)")
    ap.add_argument("--feat-policy", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap", action="store_true",
                    help="run sample -> gather -> forward of each batch back to back on one stream; by default the "
                         "sampling of batch b+1 runs on a second stream while batch b is gathered and multiplied")
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
    torch.cuda.set_device(0)
    t0 = time.time()
    indptr = torch.empty(w.num_nodes + 1, dtype=torch.int64, pin_memory=True)
    indices = torch.empty(w.num_edges, dtype=torch.int64, pin_memory=True)
    feat = torch.empty(w.num_nodes, w.feat_dim, dtype=torch.float32, pin_memory=True)
    synth.rmat_csr(w.num_nodes, w.num_edges, w.rmat, w.graph_seed, indptr_ptr=indptr.data_ptr(),
                   indices_ptr=indices.data_ptr())
    synth.features(w.num_nodes, w.feat_dim, w.feature_seed, ptr=feat.data_ptr())
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
        ctx.sync()
        t0 = time.time()
        dci.dci_presample_count(ctx, g, None, seeds, w.batch_size, 0, w.n_presample, w.presample_first_batch,
                                w.fanouts, w.rng_seed, fc, ac, feat_scratch=x, stats=stats)
        ctx.sync()
        t1 = time.time()
        st = stats.cpu().numpy()
        ts, tf = int(st[dci.STAT["t_sample_ns"]]), int(st[dci.STAT["t_feature_ns"]])
        cache = dci.dci_fill_caches(ctx, g, fc, ac, w.budget_bytes, ts, tf, args.feat_policy)
        t2 = time.time()
        pre = dict(presample_s=round(t1 - t0, 4), fill_s=round(t2 - t1, 4), t_sample_ns=ts, t_feature_ns=tf,
                   cap_adj_bytes=int(cache.cap_adj_bytes), cap_feat_bytes=int(cache.cap_feat_bytes),
                   adj_nodes=int(cache.adj_nodes), adj_edges=int(cache.adj_edges), feat_rows=int(cache.feat_rows))
        log(f"[bench] preprocess: {pre}")

    nb = w.num_batches

    # Two streams: the sampling chain of a batch is a string of short, latency-bound kernels that
    # leaves most of the chip idle, so it runs one batch ahead of the bandwidth- and MFMA-bound
    # gather / forward kernels (double-buffered blocks, events both ways).  Same default priority.
    overlap = not args.no_overlap
    s_stream = torch.cuda.Stream() if overlap else None
    ctx_s = dci.Context(0, stream=s_stream) if overlap else ctx
    blks = [blk, dci.Blocks(ctx, w.num_nodes, w.batch_size, w.fanouts)] if overlap else [blk]
    ctx_s.ensure_workspace(ctx.lib.dci_sample_workspace_bytes(w.num_nodes, w.batch_size,
                                                              (C.c_int32 * w.n_hops)(*w.fanouts), w.n_hops))

    def sample(b: int, stats_t):
        lo = (b % nb) * w.batch_size
        dci.dci_sample_khop(ctx_s, g, cache, seeds[lo:lo + w.batch_size], b % nb, w.fanouts, w.rng_seed,
                            blks[b % len(blks)], stats_t)

    def consume(b: int, stats_t):
        bk = blks[b % len(blks)]
        dci.dci_gather_features(ctx, g, cache, bk.nodes, bk.cap_nodes[-1], x, n_dev=bk.n_input_dev(), stats=stats_t)
        dci.dci_sage_forward(ctx, bk, x, ws, wn, bs, logits)

    def run_steps(first: int, count: int, stats_s, stats_c):
        """Exactly `count` whole steps (batches first .. first+count-1); nothing is in flight before or after."""
        if not overlap:
            for b in range(first, first + count):
                sample(b, stats_s)
                consume(b, stats_c)
            return
        main = torch.cuda.current_stream()
        s_stream.wait_stream(main)
        sampled = [torch.cuda.Event() for _ in range(count)]
        consumed = [torch.cuda.Event() for _ in range(count)]
        with torch.cuda.stream(s_stream):
            sample(first, stats_s)
            sampled[0].record(s_stream)
        for k in range(count):
            if k + 1 < count:
                with torch.cuda.stream(s_stream):
                    if k >= 1:
                        s_stream.wait_event(consumed[k - 1])  # the buffer of batch k+1 was last read by batch k-1
                    sample(first + k + 1, stats_s)
                    sampled[k + 1].record(s_stream)
            main.wait_event(sampled[k])
            consume(first + k, stats_c)
            consumed[k].record(main)
        main.wait_stream(s_stream)

    run_steps(0, args.warmup, None, None)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps; the dominant kernel class is bracketed by events
    dominant = "linear_in"
    ctx.timing_enable(dci.KERNEL_CLASSES if args.time_all_kernels else [dominant, "gather"])
    if args.time_all_kernels and overlap:
        ctx_s.timing_enable(dci.KERNEL_CLASSES)
    stats = torch.zeros(dci.STATS_WORDS, dtype=torch.int64, device="cuda")
    stats_s = torch.zeros(dci.STATS_WORDS, dtype=torch.int64, device="cuda") if overlap else stats
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    run_steps(0, args.steps, stats_s, stats)
    ev[1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall_s = t1 - t0
    timing = ctx.timing_read()
    ctx.timing_enable([])
    if overlap:
        for k, v in ctx_s.timing_read().items():
            timing[k] = (timing[k][0] + v[0], timing[k][1] + v[1])
        ctx_s.timing_enable([])
        stats += stats_s
    st = {k: int(v) for k, v in zip(dci.STAT.keys(), stats.cpu().numpy()[:len(dci.STAT)])}
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    edges = st["edges_sampled"]
    rows = st["feat_hits"] + st["feat_misses"]
    gather_bytes = rows * w.feat_dim * 4
    gather_ms, gather_n = timing["gather"]
    value = edges / wall_s

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
            fl = 2.0 * nn[w.n_hops - 1 - l] * (2 * w.dims[l]) * w.dims[l + 1]
            flops_all += fl
            if l == 0:
                flops_in += fl
    lin_tflops = flops_in / (lin_ms * 1e-3) / 1e12 if lin_ms > 0 else 0.0
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(f"{dominant}:{w.name}")
        except Exception:
            traffic = None
    roofline = {"kernel": "k_sage_linear (first layer)", "bound": "mfma", "achieved": round(lin_tflops, 3),
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
        ip, ix, ft = indptr.numpy(), indices.numpy(), feat.numpy()
        t0 = time.perf_counter()
        ob = oracle.sample_khop(ip, ix, seeds_h[:w.batch_size], 0, w.fanouts, w.rng_seed)
        t_s = time.perf_counter()
        ox = oracle.gather(ft, ob.nodes)
        t_g = time.perf_counter()
        ol = oracle.sage_forward(ob, ox, ws_h, wn_h, b_h)
        t_f = time.perf_counter()
        e0 = int(ob.n_edges.sum())
        cpu = {"value": round(e0 / (t_f - t0), 1), "unit": "edges/s", "cores": 1, "kind": "oracle",
               "sample": f"batch 0 of '{w.name}' ({w.batch_size} seeds, {e0} edges, {len(ob.nodes)} input nodes): "
                         f"sample {t_s - t0:.2f}s, gather {t_g - t_s:.2f}s, forward {t_f - t_g:.2f}s",
               "sample_edges_per_s": round(e0 / (t_s - t0), 1),
               "gather_GBps": round(len(ob.nodes) * w.feat_dim * 4 / (t_g - t_s) / 1e9, 3)}
        # the same batch from the GPU, as a last parity check on the benchmarked configuration
        dci.dci_sample_khop(ctx, g, cache, seeds[:w.batch_size], 0, w.fanouts, w.rng_seed, blk, None)
        dci.dci_gather_features(ctx, g, cache, blk.nodes, blk.cap_nodes[-1], x, n_dev=blk.n_input_dev())
        dci.dci_sage_forward(ctx, blk, x, ws, wn, bs, logits)
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
                   "fanouts_from_seeds": list(w.fanouts), "batch_size": w.batch_size, "dims": list(w.dims),
                   "budget_bytes": 0 if args.no_cache else w.budget_bytes, "feat_policy": args.feat_policy,
                   "cache": not args.no_cache, "overlap_sampling": overlap},
        "extras": {
            "edges_per_step": round(edges / args.steps, 1), "input_nodes_per_step": round(rows / args.steps, 1),
            "gather_GBps_delivered": round(gather_bytes / (gather_ms * 1e-3) / 1e9, 1) if gather_ms > 0 else None,
            "adj_hit_rate_edges": round(st["adj_edge_hits"] / adj_total, 4) if adj_total else None,
            "adj_hit_rate_nodes": round(st["adj_node_hits"] / max(1, st["adj_node_hits"] + st["adj_node_misses"]), 4),
            "feat_hit_rate": round(st["feat_hits"] / rows, 4) if rows else None,
            "gpu_event_ms_per_step": round(ev[0].elapsed_time(ev[1]) / args.steps, 4),
            "kernel_ms_per_step": {k: round(v[0] / args.steps, 4) for k, v in timing.items() if v[1]},
            "preprocess": pre, "gather_roofline": gather_roof,
        },
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
