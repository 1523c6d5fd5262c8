"""GPU parity at the full size of the two host-resident workloads ("huge": 111 M nodes / 1.6 B edges /
57 GB of features, "skewed": 65 M nodes / 1.8 B edges / 67 GB of features).

Placement: a GPU machine pins at most 64 GiB of host memory, less than graph + features of either workload.
The feature matrix and the list-bound array (indptr) are in pinned host memory, so feature misses and the
list bounds of adjacency misses cross the host link as in the paper's set-up; the neighbour-id array
(indices) is placed in HBM, standing in for the host tier (the kernels dereference the same kind of mapped
pointer either way).  Generating the inputs takes about two minutes per workload.

Checked: pre-sampling counters, both remaps and the compacted adjacency cache in full; cached feature rows
on 20,000 sampled rows; four consecutive batches in flight on four lanes (dci_infer_batches) through the
partially filled caches - every batch's blocks and gathered rows bit for bit, logits to 1e-4 of the
largest oracle logit - and the hit / miss / traffic statistics of those batches, exact."""
import gc
import time

import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu


def _log(msg):
    print(f"[full-scale {time.strftime('%H:%M:%S')}] {msg}", flush=True)


@pytest.mark.parametrize("name", ["huge", "skewed"])
def test_full_scale(name):
    import paper_2503_01281_amd as dci
    from tests import gpu_util as gu
    w = synth.WORKLOADS[name]
    # page-locked memory and HBM left cached by earlier tests would count against this test's 60+ GB
    gc.collect()
    torch.cuda.empty_cache()
    if hasattr(torch._C, "_host_emptyCache"):
        torch._C._host_emptyCache()
    _log(f"{name}: allocating inputs (features and indptr pinned, indices in HBM)")
    indptr = dci.pinned_empty(w.num_nodes + 1, torch.int64)
    indices_host = torch.empty(w.num_edges, dtype=torch.int64)
    feat = dci.pinned_empty(w.num_nodes * w.feat_dim, torch.float32).view(w.num_nodes, w.feat_dim)
    assert indptr.is_pinned() and feat.is_pinned()
    _log("generating graph")
    synth.rmat_csr(w.num_nodes, w.num_edges, w.rmat, w.graph_seed, indptr_ptr=indptr.data_ptr(),
                   indices_ptr=indices_host.data_ptr())
    indices = torch.empty(w.num_edges, dtype=torch.int64, device="cuda")
    for lo in range(0, w.num_edges, 1 << 27):
        indices[lo:lo + (1 << 27)].copy_(indices_host[lo:lo + (1 << 27)])
    _log("generating features")
    synth.features(w.num_nodes, w.feat_dim, w.feature_seed, ptr=feat.data_ptr())
    ft = feat.numpy()
    seeds = synth.seeds(w.num_nodes, w.num_seeds, w.seed_seed)
    ws_h, wn_h, bs_h = synth.sage_weights(w.dims, w.weight_seed)
    ip, ix = indptr.numpy(), indices_host.numpy()
    ctx = dci.Context(0)
    g = dci.Graph(indptr, indices, feat)
    seeds_dev = gu.dev(seeds)

    _log("pre-sampling (oracle)")
    fc_w, ac_w, _, (edges, nodes) = oracle.presample_count(ip, ix, seeds, w.batch_size, w.n_presample, w.fanouts,
                                                          w.rng_seed, w.presample_first_batch, with_edge_count=False)
    _log("pre-sampling (GPU, no cache: every access takes the miss path)")
    fc = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
    ac = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
    stats = gu.new_stats()
    dci.dci_presample_count(ctx, g, None, seeds_dev, w.batch_size, 0, w.n_presample, w.presample_first_batch,
                            w.fanouts, w.rng_seed, fc, ac, stats=stats)
    st = gu.stats_dict(ctx, stats)
    assert np.array_equal(fc.cpu().numpy().view(np.uint32), fc_w)
    assert np.array_equal(ac.cpu().numpy().view(np.uint32), ac_w)
    assert (st["edges_sampled"], st["input_nodes"]) == (edges, nodes)

    ts, tf = 3, 7
    _log("fill (oracle)")
    C_adj, C_feat = oracle.split(w.budget_bytes, ts, tf, w.num_nodes, w.num_edges, w.feat_dim)
    adj_remap, cp, ci = oracle.fill_adj(ip, ix, ac_w, C_adj)
    feat_remap, _, k = oracle.fill_feat(fc_w, None, C_feat, 0, feat_dim=w.feat_dim)
    _log(f"fill (GPU): C_adj={C_adj} C_feat={C_feat} K={len(cp) - 1} M={len(ci)} k={k}")
    t0 = time.time()
    cache = dci.dci_fill_caches(ctx, g, fc, ac, w.budget_bytes, ts, tf, 0)
    _log(f"fill (GPU) took {time.time() - t0:.2f}s")
    assert (cache.cap_adj_bytes, cache.cap_feat_bytes) == (C_adj, C_feat)
    assert (cache.adj_nodes, cache.adj_edges, cache.feat_rows) == (len(cp) - 1, len(ci), k)
    assert 0 < k < w.num_nodes, "the feature cache must be partial so that misses cross the host link"
    assert np.array_equal(cache.adj_remap.cpu().numpy(), adj_remap)
    assert np.array_equal(cache.feat_remap.cpu().numpy(), feat_remap)
    base = cache.buf.data_ptr()

    def view(addr, first, n, dtype):
        es = torch.tensor([], dtype=dtype).element_size()
        off = addr - base + first * es
        return cache.buf[off:off + n * es].view(dtype)

    assert np.array_equal(view(cache.c.c_indptr, 0, len(cp), torch.int64).cpu().numpy(), cp)
    chunk = 1 << 27
    for lo in range(0, len(ci), chunk):
        n = min(chunk, len(ci) - lo)
        assert np.array_equal(view(cache.c.c_indices, lo, n, torch.int64).cpu().numpy(), ci[lo:lo + n]), lo
    del ci
    rows = np.flatnonzero(feat_remap >= 0)
    pick = rows[np.random.default_rng(0).integers(0, len(rows), 20000)]
    slots = torch.from_numpy(feat_remap[pick].astype(np.int64)).cuda()
    got_rows = view(cache.c.feat_cache, 0, k * w.feat_dim, torch.float32).view(k, w.feat_dim)[slots].cpu().numpy()
    assert got_rows.tobytes() == ft[pick].tobytes()
    _log("caches match")

    # four consecutive batches in flight on four lanes
    ws, wn, bs = ([gu.dev(a) for a in arr] for arr in (ws_h, wn_h, bs_h))
    lanes = [dci.Lane(g, w.batch_size, w.fanouts, w.dims) for _ in range(4)]
    first = 1
    logits = torch.full((w.num_seeds, w.classes), float("nan"), dtype=torch.float32, device="cuda")
    stats = gu.new_stats()
    torch.cuda.synchronize()
    dci.dci_infer_batches(lanes, g, cache, seeds_dev, w.batch_size, first, 4, w.fanouts, w.rng_seed, 0, ws, wn, bs,
                          logits, stats)
    for ln in lanes:
        ln.ctx.sync()
    st = gu.stats_dict(ctx, stats)
    tot = dict(edges=0, nodes=0, feat_hits=0, adj_hit_edges=0, adj_hit_nodes=0, rows=0)
    for k_, ln in enumerate(lanes):
        b = first + k_
        sl = slice(b * w.batch_size, (b + 1) * w.batch_size)
        _log(f"batch {b} (oracle)")
        want = oracle.sample_khop(ip, ix, seeds[sl], b, w.fanouts, w.rng_seed)
        gu.assert_blocks_equal(gu.blocks_to_host(ln.ctx, ln.blocks), want)
        want_x = oracle.gather(ft, want.nodes)
        assert ln.x[:len(want.nodes)].cpu().numpy().tobytes() == want_x.tobytes()
        ref = oracle.sage_forward(want, want_x, ws_h, wn_h, bs_h)
        err = float(np.abs(logits[sl].cpu().numpy() - ref).max())
        assert err <= 1e-4 * max(1.0, float(np.abs(ref).max())), err
        tot["edges"] += int(want.n_edges.sum())
        tot["nodes"] += len(want.nodes)
        tot["feat_hits"] += int((feat_remap[want.nodes] >= 0).sum())
        for h in range(w.n_hops):
            hit = adj_remap[want.nodes[:want.n_nodes[h]]] >= 0
            tot["adj_hit_edges"] += int(np.diff(want.blk_indptr[h])[hit].sum())
            tot["adj_hit_nodes"] += int(hit.sum())
            tot["rows"] += int(want.n_nodes[h])
        _log(f"{name}: batch {b} matches: {int(want.n_edges.sum())} edges, {len(want.nodes)} input nodes, "
             f"max logit error {err:.2e}")
    assert (st["edges_sampled"], st["input_nodes"]) == (tot["edges"], tot["nodes"])
    assert (st["feat_hits"], st["feat_misses"]) == (tot["feat_hits"], tot["nodes"] - tot["feat_hits"])
    assert st["feat_misses"] > 0
    assert (st["adj_edge_hits"], st["adj_node_hits"]) == (tot["adj_hit_edges"], tot["adj_hit_nodes"])
    F4 = 4 * w.feat_dim
    assert st["bytes_hbm"] == 16 * tot["adj_hit_nodes"] + 8 * tot["adj_hit_edges"] + F4 * tot["feat_hits"]
    assert st["bytes_host"] == (16 * (tot["rows"] - tot["adj_hit_nodes"]) + 8 * (tot["edges"] - tot["adj_hit_edges"])
                                + F4 * (tot["nodes"] - tot["feat_hits"]))
    _log(f"{name}: feature hit rate {tot['feat_hits'] / tot['nodes']:.4f}, adjacency edge hit rate "
         f"{tot['adj_hit_edges'] / max(1, tot['edges']):.4f}, host bytes per batch {st['bytes_host'] / 4 / 1e6:.1f} MB")
