#!/usr/bin/env python3
"""Benchmark of the dual-cache GNN inference hot path on one MI355X.

A step is one pass of the per-batch path (cache-aware k-hop sampling -> cache-aware feature
gather -> GraphSAGE-mean forward) over one mini-batch of the workload; the one-off part of the
path (pre-sampling counts, Eq. (1) split with the stage times measured while pre-sampling,
dual-cache fill) runs before the timed region and is reported separately.  Inputs are seeded
synthetic R-MAT graphs / Gaussian features / Glorot weights with the shapes of the paper's
datasets, resident in pinned host memory (graph, features) and HBM (caches, seeds, weights) when
the timed region starts.  The default workload is the largest single-GPU configuration ("huge",
the shape of Ogbn-papers100M with a 64 GB budget).

Regions, in order (all over the same K batches 0..K-1):
  warm-up        W steps, untimed;
  kernel pass    K steps, untimed, with every kernel class bracketed by HIP events on the
                 library's stream -> extras.rooflines (one entry per class: algorithmic bytes /
                 flops from the batches' own device-side sizes against the bound that applies)
                 and the choice of the dominant kernel (largest average launch);
  timed region   EXACTLY K steps on one stream (one lane of dci_infer_batches) with only the
                 dominant class bracketed -> value, ms_per_step, roofline;
  pipelined      the same K steps with `--lanes` batches in flight -> extras.pipelined;
  end to end     pre-sampling + fill + one pass over ALL batches of the workload, pipelined,
                 measured wall time -> extras.end_to_end;
  memory rates   streaming and random reads of HBM and of pinned host memory (dci_probe_read) and
                 a pinned host -> HBM copy -> extras.memory_rates (the measured denominators);
  cpu_baseline   the CPU oracle on this machine's host cores on a bounded sample (one thread,
                 then one thread per core over independent batches), and a parity check of the
                 benchmarked batch 0 against it.

Prints ONE JSON line.
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

HBM_PEAK_GBPS = 8000.0
FP32_MFMA_PEAK_TFLOPS = 157.3
PIN_LIMIT_BYTES = 60 * 10**9     # the GPU machines refuse page-locked allocations beyond 64 GiB in total


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="huge", choices=["tiny", "medium", "large", "huge", "skewed", "yelp", "amazon"])
    ap.add_argument("--placement", default="auto", choices=["auto", "host", "indices-hbm", "features-hbm"],
                    help="where the graph and the features live: 'host' = all in pinned host memory; 'indices-hbm' = "
                         "features and list bounds pinned, neighbour ids in HBM; 'features-hbm' = graph pinned, features "
                         "in HBM; 'auto' = 'host' when graph + features fit the pinned-memory limit, else 'indices-hbm'")
    ap.add_argument("--no-cache", action="store_true", help="run the miss path only (no dual cache)")
    ap.add_argument("--feat-policy", type=int, default=0)
    ap.add_argument("--budget", type=float, default=None, help="cache budget in bytes (default: the workload's)")
    ap.add_argument("--n-presample", type=int, default=None, help="pre-sampled batches (default: the workload's 8)")
    ap.add_argument("--split-times", default=None, metavar="TS:TF",
                    help="fixed t_sample:t_feature for Eq. (1) instead of the times measured while pre-sampling")
    ap.add_argument("--single-cache", action="store_true",
                    help="the paper's single-cache comparison: the whole budget goes to features, no adjacency cache")
    ap.add_argument("--adj-elements", action="store_true",
                    help="element-granular adjacency cache (Algorithm 1 as printed): lists reordered by element count, "
                         "last node cached in part; pre-sampling then also counts per element")
    ap.add_argument("--model", default="sage-mean", choices=["sage-mean", "sage-sum", "gcn-avg"],
                    help="GNN of the forward pass (Table III); the headline configuration is sage-mean")
    ap.add_argument("--linear-kernel", type=int, default=0, choices=[0, 1, 2, 3, 4],
                    help="dense-layer kernel of the single-stream regions: 0 by shape (default), 1 register-staged tile "
                         "kernel, 2 wide kernel, 3 by shape without the wide and the weights-in-registers kernels, "
                         "4 weights in registers where the shape allows")
    ap.add_argument("--pipelined-linear-kernel", type=int, default=1, choices=[0, 1, 2, 3, 4],
                    help="dense-layer kernel of the pipelined regions (the statically partitioned wide kernel loses "
                         "when other streams share the compute units)")
    ap.add_argument("--fused-input", type=int, default=1, choices=[0, 1],
                    help="1 (default): the input layer reads cached neighbour rows in place (dci_gather_forward: only "
                         "missed rows and the rows of F_{L-1} are copied); 0: dci_gather_features then dci_gnn_forward")
    ap.add_argument("--input-layer", type=int, default=0, choices=[0, 1, 2, 3],
                    help="first layer: 0 (default) one kernel (aggregation inside the dense layer) where the layer is "
                         "large enough and its shape allows one of the two forms, 1 always aggregation kernel + dense kernel, "
                         "2 / 3 the one-kernel form wherever the shape allows (weights in registers / 64-row tiles)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-batches", type=int, default=None, help="batches the single-thread CPU oracle is timed on")
    ap.add_argument("--lanes", type=int, default=4, help="batches in flight in the pipelined regions (0 or 1 = skip them)")
    ap.add_argument("--lanes-sweep", default=None, metavar="N,N,...",
                    help="also time the pipelined region with these lane counts and dense-layer kernels 0, 1, 3 and 4 "
                         "(extras.pipelined_sweep)")
    ap.add_argument("--roofline-kernel", default="auto",
                    help="kernel class of the top-level roofline (default: the one with the largest average launch in "
                         "the kernel pass)")
    ap.add_argument("--no-end-to-end", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="at the end run one device-to-device copy of 1 GiB (a kernel of known traffic for scaling "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE)")
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
    # those the feature matrix and the list-bound array stay pinned and the neighbour-id array is placed in HBM,
    # standing in for the host tier.
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
        f"(N={w.num_nodes} E={w.num_edges} F={w.feat_dim}, placement {place})")

    model = {"sage-mean": 0, "sage-sum": 1, "gcn-avg": 2}[args.model]
    k_ops = 1 if model == 2 else 2      # operands of the dense layer's contraction (GCN has one weight matrix)
    g = dci.Graph(indptr, indices, feat)
    seeds = torch.from_numpy(seeds_h).cuda()
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    ws, wn, bs = [dev(a) for a in ws_h], [dev(a) for a in wn_h], [dev(a) for a in b_h]
    ws_arg = None if model == 2 else ws
    sweep = [int(v) for v in args.lanes_sweep.split(",")] if args.lanes_sweep else []
    n_lanes = max([1, args.lanes] + sweep)
    # lane 0 runs on PyTorch's current stream (the single-stream regions); the others on streams of their own,
    # all at the default priority
    lanes = [dci.Lane(g, w.batch_size, w.fanouts, w.dims, stream=torch.cuda.current_stream() if k == 0 else None)
             for k in range(n_lanes)]
    ctx, blk, x = lanes[0].ctx, lanes[0].blocks, lanes[0].x
    nb = w.num_batches
    logits = torch.empty(w.num_seeds, w.classes, dtype=torch.float32, device="cuda")
    for ln in lanes:
        ln.ctx.set_option(dci.DCI_OPT_FUSED_INPUT, args.fused_input)
        ln.ctx.set_option(dci.DCI_OPT_INPUT_LAYER, args.input_layer)

    # ---- one-off part: pre-sampling counts (timed per stage for Eq. (1)) and the dual-cache fill
    cache = None
    pre = {}
    if not args.no_cache:
        fc = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
        ac = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
        stats = torch.zeros(dci.STATS_WORDS, dtype=torch.int64, device="cuda")
        ec = torch.zeros(w.num_edges, dtype=torch.int32, device="cuda") if args.adj_elements else None
        fill_flags = args.feat_policy | (dci.DCI_FILL_ADJ_ELEMENTS if args.adj_elements else 0)
        torch.cuda.synchronize()
        t0 = time.time()
        dci.dci_presample_count(ctx, g, None, seeds, w.batch_size, 0, w.n_presample, w.presample_first_batch,
                                w.fanouts, w.rng_seed, fc, ac, ec, feat_scratch=x, stats=stats)
        ctx.sync()
        t1 = time.time()
        st = stats.cpu().numpy()
        ts, tf = int(st[dci.STAT["t_sample_ns"]]), int(st[dci.STAT["t_feature_ns"]])
        ts_used, tf_used = ts, tf
        if args.split_times:
            ts_used, tf_used = (int(v) for v in args.split_times.split(":"))
        if args.single_cache:
            cache = dci.dci_fill_caches(ctx, g, fc, ac, w.budget_bytes, 0, 1, fill_flags | dci.DCI_FILL_STRICT_SPLIT,
                                        edge_count=ec)
        else:
            cache = dci.dci_fill_caches(ctx, g, fc, ac, w.budget_bytes, ts_used, tf_used, fill_flags, edge_count=ec)
        del ec
        t2 = time.time()
        if args.adj_elements and indices_host is not indices:
            # the element-granular fill reordered the lists in place (in HBM here): the oracle must see the same lists
            for lo_ in range(0, w.num_edges, 1 << 27):
                indices_host[lo_:lo_ + (1 << 27)].copy_(indices[lo_:lo_ + (1 << 27)])
        pre = dict(presample_s=round(t1 - t0, 4), fill_s=round(t2 - t1, 4), t_sample_ns=ts, t_feature_ns=tf,
                   split_times="measured" if not args.split_times else args.split_times,
                   cap_adj_bytes=int(cache.cap_adj_bytes), cap_feat_bytes=int(cache.cap_feat_bytes),
                   adj_nodes=int(cache.adj_nodes), adj_edges=int(cache.adj_edges), feat_rows=int(cache.feat_rows),
                   adj_elements=bool(args.adj_elements), adj_partial_node=int(cache.adj_partial_node))
        log(f"[bench] preprocess: {pre}")
    torch.cuda.synchronize()

    def run(first: int, count: int, use_lanes: int, stats_t=None):
        """Batches first .. first+count-1 on the first `use_lanes` lanes; returns when all of them are done."""
        dci.dci_infer_batches(lanes[:use_lanes], g, cache, seeds, w.batch_size, first, count, w.fanouts, w.rng_seed,
                              model, ws_arg, wn, bs, logits, stats_t)
        for ln in lanes[:use_lanes]:
            ln.ctx.sync()

    K = min(args.steps, nb)
    if K < args.steps:
        log(f"[bench] the workload has {nb} batches: timing {K} steps instead of {args.steps}")
    ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, args.linear_kernel)
    run(0, min(args.warmup, nb), 1)

    # ---- kernel pass: every class bracketed; per-hop sizes of every batch from the device-side counts
    ctx.timing_enable(dci.KERNEL_CLASSES)
    stats_k = torch.zeros(dci.STATS_WORDS, dtype=torch.int64, device="cuda")
    hop_nodes = np.zeros(w.n_hops + 1, dtype=np.int64)
    hop_edges = np.zeros(w.n_hops, dtype=np.int64)
    flops_layer = np.zeros(w.n_hops)
    for b in range(K):
        run(b, 1, 1, stats_k)
        nn, ne = blk.n_nodes(), blk.n_edges()
        hop_nodes += np.array(nn, dtype=np.int64)
        hop_edges += np.array(ne, dtype=np.int64)
        for l in range(w.n_hops):
            flops_layer[l] += 2.0 * nn[w.n_hops - 1 - l] * (k_ops * w.dims[l]) * w.dims[l + 1]
    timing_all = ctx.timing_read()
    ctx.timing_enable([])
    sk = {k: int(v) for k, v in zip(dci.STAT.keys(), stats_k.cpu().numpy()[:len(dci.STAT)])}

    # ---- memory rates measured in this run (the denominators of the access-bound kernels)
    rates = {}
    probe_dev = cache.buf if cache is not None else torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    dev_bytes = min(probe_dev.numel() - 512, 8 << 30)
    host_t = feat if feat.is_pinned() else indices
    host_bytes = min(host_t.numel() * host_t.element_size() - 512, 2 << 30)

    def probe(mem, nbytes, granule, n):
        dci.dci_probe_read(ctx, mem, granule, n, 0, 4096, 11, nbytes)
        return min(dci.dci_probe_read(ctx, mem, granule, n, 0, 4096, 12 + r, nbytes) for r in range(2))

    rates["hbm_stream_read_GBps"] = round(dev_bytes / probe(probe_dev, dev_bytes, 0, 0) / 1e6, 1)
    for gran in (8, 64, 128):
        rates[f"hbm_random_{gran}B_Gacc_per_s"] = round((1 << 25) / probe(probe_dev, dev_bytes, gran, 1 << 25) / 1e6, 2)
    rates["host_zero_copy_stream_GBps"] = round(host_bytes / probe(host_t, host_bytes, 0, 0) / 1e6, 1)
    for gran in (8, 64, 128, 512):
        rates[f"host_zero_copy_random_{gran}B_Gacc_per_s"] = round((1 << 20) / probe(host_t, host_bytes, gran, 1 << 20) / 1e6, 4)
    flat = host_t.view(-1)
    n_link = min(flat.numel(), (1 << 30) // flat.element_size())
    link_dst = torch.empty(n_link, dtype=flat.dtype, device="cuda")
    link_ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    link_dst.copy_(flat[:n_link], non_blocking=True)
    torch.cuda.synchronize()
    link_ev[0].record()
    link_dst.copy_(flat[:n_link], non_blocking=True)
    link_ev[1].record()
    torch.cuda.synchronize()
    host_link_gbps = n_link * flat.element_size() / (link_ev[0].elapsed_time(link_ev[1]) * 1e-3) / 1e9
    rates["host_pinned_copy_GBps"] = round(host_link_gbps, 1)
    del link_dst
    # Host-link ceilings.  Small reads: a request of up to 128 bytes costs the same whatever it carries, so the
    # sampler's misses are charged in 128-byte lines; no access pattern moves lines faster than a streaming read,
    # which is the peak used (isolated random lines go at `random_line_rate`, adjacent ones merge into larger
    # requests and go faster).  Feature rows: the pinned-copy rate.
    random_line_rate = rates["host_zero_copy_random_128B_Gacc_per_s"] * 1e9
    line_rate = rates["host_zero_copy_stream_GBps"] * 1e9 / 128.0
    row_link_rate = host_link_gbps * 1e9
    hbm_bw = HBM_PEAK_GBPS * 1e9

    # ---- per-class rooflines from the kernel pass (units per SURVEY-style accounting, stated in the design doc):
    #   sampling  28 B per frontier node (id, remap, list bounds) + 16 B per edge (id read, id written);
    #             what a miss reads from pinned host memory is charged in 128-byte lines over the link
    #   relabel   20 B per edge (table probe + local id) + 8 B per new node        gather  8F+12 B per row
    #   mean      4D B per edge + 4D B per destination row                         linear  2 n (k D) D' flop
    F, L = w.feat_dim, w.n_hops
    rows_total = int(hop_nodes[:L].sum())
    edges_total = int(hop_edges.sum())
    n_in_total = int(hop_nodes[L])
    miss_rows = rows_total - sk["adj_node_hits"]
    link_lines = (sk["lines_bounds"] if indptr.is_pinned() else 0) + (sk["lines_ids"] if indices.is_pinned() else 0)
    link_bytes_sampler = (16 * miss_rows if indptr.is_pinned() else 0) + (8 * sk["adj_edge_misses"] if indices.is_pinned() else 0)
    table_entries = max(1024, 2 * blk.cap_nodes[L])     # the sampler's per-batch hash table: 8 bytes per entry

    def entry(kernel, cls, t_bound_parts, achieved, peak, unit, **more):
        """t_bound_parts: {bound name: seconds that bound allows}; the largest one is the class's bound."""
        t_ms, n = timing_all[cls]
        bound = max(t_bound_parts, key=t_bound_parts.get)
        t_bound = t_bound_parts[bound]
        d = {"kernel": kernel, "bound": bound, "achieved": None, "peak": None, "unit": unit[bound],
             "frac": round(t_bound / (t_ms * 1e-3), 4) if t_ms > 0 else None,
             "ms_per_step": round(t_ms / K, 4), "launches_per_step": round(n / K, 2)}
        if t_ms > 0:
            d["achieved"] = round(achieved[bound] / (t_ms * 1e-3), 3)
            d["peak"] = round(peak[bound], 3)
        d.update(more)
        return d

    GB, unit_hbm = 1e9, {"hbm": "GB/s", "host_link": "G lines/s", "host_link_bytes": "GB/s", "mfma": "TFLOP/s"}
    rooflines = {}
    clear_bytes = 8 * table_entries * K
    rooflines["table_clear"] = entry("k_fill_u32x4", "table_clear", {"hbm": clear_bytes / hbm_bw}, {"hbm": clear_bytes / GB},
                                     {"hbm": HBM_PEAK_GBPS}, unit_hbm, bytes_per_step=8 * table_entries)
    samp_hbm = 28 * rows_total + 16 * edges_total - link_bytes_sampler
    rooflines["sample"] = entry("k_sample_hop", "sample",
                                {"hbm": samp_hbm / hbm_bw, "host_link": link_lines / line_rate if line_rate else 0.0},
                                {"hbm": samp_hbm / GB, "host_link": link_lines / 1e9},
                                {"hbm": HBM_PEAK_GBPS, "host_link": line_rate / 1e9}, unit_hbm,
                                hbm_bytes_per_step=round(samp_hbm / K), host_lines_per_step=round(link_lines / K, 1),
                                host_bytes_per_step=round(link_bytes_sampler / K),
                                frontier_nodes_per_step=round(rows_total / K, 1),
                                host_lines_vs_random_line_rate=(round(link_lines / (timing_all["sample"][0] * 1e-3) / random_line_rate, 4)
                                                                if timing_all["sample"][0] > 0 and random_line_rate else None))
    relabel_bytes = 20 * edges_total + 8 * int(hop_nodes[L] - hop_nodes[0])
    t_rl = timing_all["relabel"][0] + timing_all["write_src"][0]
    timing_all["relabel+write_src"] = (t_rl, timing_all["relabel"][1] + timing_all["write_src"][1])
    rooflines["relabel"] = entry("k_relabel_hop + k_write_src", "relabel+write_src", {"hbm": relabel_bytes / hbm_bw},
                                 {"hbm": relabel_bytes / GB}, {"hbm": HBM_PEAK_GBPS}, unit_hbm,
                                 bytes_per_step=round(relabel_bytes / K))
    # gather: 8F+12 B per row that is copied (4F of them over the link on a miss), 16 B (id, remap, slot note) per row
    # that is left in the cache for the input layer to read in place
    copied_hits = sk["rows_copied"] - sk["feat_misses"]
    g_hbm = (copied_hits * (8 * F + 12) + sk["feat_misses"] * ((4 * F + 12) if feat.is_pinned() else (8 * F + 12))
             + (sk["feat_hits"] - copied_hits) * 16)
    g_link = sk["feat_misses"] * 4 * F if feat.is_pinned() else 0
    rooflines["gather"] = entry("k_gather" + (" (misses and F_{L-1} rows only)" if args.fused_input else ""), "gather",
                                {"hbm": g_hbm / hbm_bw, "host_link_bytes": g_link / row_link_rate if row_link_rate else 0.0},
                                {"hbm": g_hbm / GB, "host_link_bytes": g_link / GB},
                                {"hbm": HBM_PEAK_GBPS, "host_link_bytes": row_link_rate / GB}, unit_hbm,
                                hbm_bytes_per_step=round(g_hbm / K), host_bytes_per_step=round(g_link / K),
                                rows_per_step=round(n_in_total / K, 1))
    for l in range(L):
        h = L - 1 - l
        cls_m, cls_l = ("mean_in", "linear_in") if l == 0 else ("mean", "linear")
        mb = 4 * w.dims[l] * (int(hop_edges[h]) + int(hop_nodes[h])) + (4 * int(hop_edges[h]) if l == 0 and args.fused_input else 0)
        if l <= 1:
            if l == 1 and L > 2:       # the later layers share one class: add them up
                mb = sum(4 * w.dims[j] * (int(hop_edges[L - 1 - j]) + int(hop_nodes[L - 1 - j])) for j in range(1, L))
            fl = flops_layer[0] if l == 0 else float(flops_layer[1:].sum())
            one_kernel = l == 0 and timing_all[cls_m][1] == 0 and timing_all[cls_l][1] > 0
            if one_kernel:
                # the input layer ran as one kernel (aggregation inside the dense layer): it answers to both bounds
                rooflines[cls_l] = entry("k_sage_input_res / k_sage_input_tile (aggregation inside the dense layer)", cls_l,
                                         {"hbm": mb / hbm_bw, "mfma": fl / (FP32_MFMA_PEAK_TFLOPS * 1e12)},
                                         {"hbm": mb / GB, "mfma": fl / 1e12},
                                         {"hbm": HBM_PEAK_GBPS, "mfma": FP32_MFMA_PEAK_TFLOPS}, unit_hbm,
                                         bytes_per_step=round(mb / K), flops_per_step=round(fl / K))
                continue
            rooflines[cls_m] = entry("k_sage_mean", cls_m, {"hbm": mb / hbm_bw}, {"hbm": mb / GB}, {"hbm": HBM_PEAK_GBPS},
                                     unit_hbm, bytes_per_step=round(mb / K))
            rooflines[cls_l] = entry("dense layer (fp32 MFMA)", cls_l, {"mfma": fl / (FP32_MFMA_PEAK_TFLOPS * 1e12)},
                                     {"mfma": fl / 1e12}, {"mfma": FP32_MFMA_PEAK_TFLOPS}, unit_hbm,
                                     flops_per_step=round(fl / K))
    if args.fused_input and timing_all["mean_in"][1] > 0:
        # the pair against what the two separate steps are defined to move: every input row gathered (8F+12 B on a
        # hit) and every edge's row read once more for the aggregate
        full = (sk["feat_hits"] * (8 * F + 12) + sk["feat_misses"] * ((4 * F + 12) if feat.is_pinned() else (8 * F + 12))
                + 4 * F * (int(hop_edges[L - 1]) + int(hop_nodes[L - 1])))
        timing_all["gather+mean_in"] = (timing_all["gather"][0] + timing_all["mean_in"][0],
                                        timing_all["gather"][1] + timing_all["mean_in"][1])
        rooflines["gather+mean_in"] = entry("k_gather + k_sage_mean (input layer, cached rows read in place)", "gather+mean_in",
                                            {"hbm": full / hbm_bw, "host_link_bytes": g_link / row_link_rate if row_link_rate else 0.0},
                                            {"hbm": full / GB, "host_link_bytes": g_link / GB},
                                            {"hbm": HBM_PEAK_GBPS, "host_link_bytes": row_link_rate / GB}, unit_hbm,
                                            note="bytes of the unfused definition (gather every row, then aggregate) over the "
                                                 "time of the fused pair")
    avg_launch = {c: (timing_all[c][0] / timing_all[c][1]) for c in dci.KERNEL_CLASSES if timing_all[c][1]}
    dominant = args.roofline_kernel if args.roofline_kernel != "auto" else max(avg_launch, key=avg_launch.get)
    roof_key = {"write_src": "relabel"}.get(dominant, dominant)

    # ---- timed region: exactly K steps, one stream, only the dominant class bracketed
    # (statistics are optional instrumentation and are left out here: the hit rates and the edge count of these
    # same K batches come from the kernel pass)
    ctx.timing_enable([dominant])
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    run(0, K, 1, None)
    ev[1].record()
    torch.cuda.synchronize()
    wall_s = time.perf_counter() - t0
    dom_ms, dom_n = ctx.timing_read()[dominant]
    ctx.timing_enable([])
    st = sk
    edges = st["edges_sampled"]
    rows = st["feat_hits"] + st["feat_misses"]
    value = edges / wall_s

    # the top-level roofline: the dominant class with the timed region's own event times
    r0 = dict(rooflines[roof_key])
    if dominant == roof_key:
        scale = (timing_all[dominant][0] / dom_ms) if dom_ms > 0 else 0.0
        r0["achieved"] = round(r0["achieved"] * scale, 3) if r0["achieved"] is not None else None
        r0["frac"] = round(r0["frac"] * scale, 4) if r0["frac"] is not None else None
    roofline = {"kernel": r0["kernel"], "bound": r0["bound"], "achieved": r0["achieved"], "peak": r0["peak"],
                "unit": r0["unit"], "frac": r0["frac"], "traffic": None, "traffic_source": None, "launches": dom_n,
                "avg_launch_ms": round(dom_ms / max(dom_n, 1), 4), "class": dominant}
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath) and model == 0:
        try:
            roofline["traffic"] = json.load(open(tpath)).get(f"{dominant}:{w.name}")
            if roofline["traffic"] is not None:
                roofline["traffic_source"] = "profiles/traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, not measured in this run)"
        except Exception:
            pass

    # ---- pipelined: the same K steps with several batches in flight
    pipelined = None
    if args.lanes > 1:
        for ln in lanes:
            ln.ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, args.pipelined_linear_kernel)
        run(0, min(K, 2 * args.lanes), args.lanes)
        torch.cuda.synchronize()
        tm0 = time.perf_counter()
        run(0, K, args.lanes)
        torch.cuda.synchronize()
        tm = time.perf_counter() - tm0
        pipelined = {"lanes": args.lanes, "linear_kernel": args.pipelined_linear_kernel, "ms_per_step": round(tm * 1e3 / K, 4),
                     "value": round(edges / tm, 1)}

    pipelined_sweep = None
    if sweep:
        pipelined_sweep = []
        for nl in sweep:
            for lk in (0, 1, 3, 4):
                for ln in lanes:
                    ln.ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, lk)
                run(0, min(K, 2 * nl), nl)
                torch.cuda.synchronize()
                tm0 = time.perf_counter()
                run(0, K, nl)
                torch.cuda.synchronize()
                tm = time.perf_counter() - tm0
                pipelined_sweep.append({"lanes": nl, "linear_kernel": lk, "ms_per_step": round(tm * 1e3 / K, 4)})
        log(f"[bench] pipelined sweep: {pipelined_sweep}")

    # ---- end to end: pre-sampling + fill (measured above) + one pass over all batches, pipelined, wall time
    e2e = None
    if not args.no_end_to_end:
        use = max(1, args.lanes)
        for ln in lanes:
            ln.ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, args.pipelined_linear_kernel if use > 1 else args.linear_kernel)
        torch.cuda.synchronize()
        te0 = time.perf_counter()
        run(0, nb, use)
        torch.cuda.synchronize()
        te = time.perf_counter() - te0
        e2e = {"batches": nb, "lanes": use, "inference_s": round(te, 4), "presample_s": pre.get("presample_s"),
               "fill_s": pre.get("fill_s"),
               "total_s": round(te + (pre.get("presample_s") or 0.0) + (pre.get("fill_s") or 0.0), 4)}
    for ln in lanes:
        ln.ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, args.linear_kernel)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- CPU oracle on this machine's host cores, bounded sample
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        ip, ix, ft = indptr.numpy(), indices_host.numpy(), feat_host.numpy()
        # sized for about 10-30 s of CPU work: the forward pass dominates, ~2 s per batch on the large workloads
        n_cpu = args.cpu_batches if args.cpu_batches is not None else (8 if w.name in ("tiny", "medium") else 4)
        n_cpu = max(1, min(n_cpu, nb))
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
               "sample": f"batches 0..{n_cpu - 1} of '{w.name}' ({e_cpu} edges, {rows_cpu} input rows) on one thread: "
                         f"sample {t_s:.2f}s, gather {t_g:.2f}s, forward {t_f:.2f}s",
               "sample_edges_per_s": round(e_cpu / t_s, 1),
               "gather_GBps": round(rows_cpu * w.feat_dim * 4 / t_g / 1e9, 3)}
        # second leg: one thread per core over independent batches (the sampler's RNG is counter-based)
        threads = max(1, min(16, len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)))
        n_all = min(nb, 2 * threads)
        r = oracle.run_batches(ip, ix, ft, seeds_h, w.batch_size, 0, n_all, w.fanouts, w.rng_seed, model,
                               None if model == 2 else ws_h, wn_h, b_h, n_threads=threads)
        cpu_model = ""
        try:
            for line in open("/proc/cpuinfo"):
                if line.startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
        except OSError:
            pass
        cpu["all_cores"] = {"value": round(r["edges"] / r["wall_s"], 1), "unit": "edges/s", "cores": min(threads, r["batches"]),
                            "cpu_model": cpu_model,
                            "sample": f"batches 0..{r['batches'] - 1}, batch k on thread k mod {threads} ({r['edges']} edges): "
                                      f"wall {r['wall_s']:.2f}s; thread-seconds sample {r['sample_s']:.2f}, gather "
                                      f"{r['gather_s']:.2f}, forward {r['forward_s']:.2f}",
                            "sample_edges_per_s": round(r["edges"] / (r["sample_s"] / min(threads, r["batches"])), 1),
                            "gather_GBps": round(r["input_rows"] * w.feat_dim * 4 / (r["gather_s"] / min(threads, r["batches"])) / 1e9, 3)}
        # the same batch from the GPU, as a last parity check on the benchmarked configuration
        run(0, 1, 1)
        nn = blk.n_nodes()
        ok_nodes = nn == [int(v) for v in ob.n_nodes] and bool(np.array_equal(blk.nodes[:nn[-1]].cpu().numpy(), ob.nodes))
        ok_src = all(np.array_equal(blk.blk_src[h][:blk.n_edges()[h]].cpu().numpy(), ob.blk_src[h]) for h in range(w.n_hops))
        dci.dci_gather_features(ctx, g, cache, blk.nodes, blk.cap_nodes[-1], x, n_dev=blk.n_input_dev())
        ctx.sync()
        ok_x = x[:nn[-1]].cpu().numpy().tobytes() == ox.tobytes()
        err = float(np.abs(logits[:w.batch_size].cpu().numpy() - ol).max())
        tol = 1e-4 * max(1.0, float(np.abs(ol).max()))
        cpu["parity"] = {"blocks_bit_exact": bool(ok_nodes and ok_src), "features_bit_exact": bool(ok_x),
                         "max_logit_err": err, "logit_tol": tol, "ok": bool(ok_nodes and ok_src and ok_x and err <= tol)}

    adj_total = st["adj_edge_hits"] + st["adj_edge_misses"]
    gather_ms = timing_all["gather"][0]
    out = {
        "metric": "sampled edges/s through sample+gather+forward (gathered feature GB/s, fractions of the HBM / host-link "
                  "rooflines and cache hit rates in extras)",
        "value": round(value, 1), "unit": "edges/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": round(wall_s * 1e3 / K, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "nodes": w.num_nodes, "edges": w.num_edges, "feat_dim": w.feat_dim,
                   "fanouts_from_seeds": list(w.fanouts), "batch_size": w.batch_size, "sage_dims": list(w.dims), "gnn": args.model,
                   "budget_bytes": 0 if args.no_cache else w.budget_bytes, "feat_policy": args.feat_policy,
                   "n_presample": w.n_presample, "single_cache": bool(args.single_cache),
                   "adj_elements": bool(args.adj_elements), "cache": not args.no_cache, "streams": 1,
                   "fused_input": bool(args.fused_input),
                   "placement": place, "features": "hbm" if feat_in_hbm else "pinned host",
                   "indices": "hbm (stand-in for the host tier: a box pins at most 64 GiB)" if place == "indices-hbm" else "pinned host",
                   "indptr": "pinned host"},
        "extras": {
            "edges_per_step": round(edges / K, 1), "input_nodes_per_step": round(rows / K, 1),
            "gather_GBps_delivered": round(n_in_total * 4 * F / (gather_ms * 1e-3) / 1e9, 1) if gather_ms > 0 else None,
            "adj_hit_rate_edges": round(st["adj_edge_hits"] / adj_total, 4) if adj_total else None,
            "adj_hit_rate_nodes": round(st["adj_node_hits"] / max(1, st["adj_node_hits"] + st["adj_node_misses"]), 4),
            "feat_hit_rate": round(st["feat_hits"] / rows, 4) if rows else None,
            "bytes_from_caches_per_step": round(st["bytes_hbm"] / K), "bytes_from_graph_arrays_per_step": round(st["bytes_host"] / K),
            "gpu_event_ms_per_step": round(ev[0].elapsed_time(ev[1]) / K, 4),
            "kernel_pass_ms_per_step": {k: round(v[0] / K, 4) for k, v in timing_all.items() if v[1] and "+" not in k},
            "rows_copied_by_gather_per_step": round(sk["rows_copied"] / K, 1),
            "rooflines": rooflines, "memory_rates": rates,
            "preprocess": pre, "pipelined": pipelined, "pipelined_sweep": pipelined_sweep, "end_to_end": e2e,
        },
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
