"""GPU parity at the full sizes of the medium and large workloads, in the launch configuration that
bench.py times: counters, remaps and cache arrays in full, two whole batches bit for bit (logits to
1e-4 of the largest oracle logit), with the configured budget and with a budget small enough that
both caches are partial."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu


def _setup(name):
    import paper_2503_01281_amd as dci
    from tests import gpu_util as gu
    w = synth.WORKLOADS[name]
    indptr = torch.empty(w.num_nodes + 1, dtype=torch.int64, pin_memory=True)
    indices = torch.empty(w.num_edges, dtype=torch.int64, pin_memory=True)
    feat = torch.empty(w.num_nodes, w.feat_dim, dtype=torch.float32, pin_memory=True)
    synth.rmat_csr(w.num_nodes, w.num_edges, w.rmat, w.graph_seed, indptr_ptr=indptr.data_ptr(),
                   indices_ptr=indices.data_ptr())
    synth.features(w.num_nodes, w.feat_dim, w.feature_seed, ptr=feat.data_ptr())
    seeds = synth.seeds(w.num_nodes, w.num_seeds, w.seed_seed)
    ws, wn, bs = synth.sage_weights(w.dims, w.weight_seed)
    ctx = dci.Context(0)
    g = dci.Graph(indptr, indices, feat)
    return dict(dci=dci, gu=gu, w=w, ctx=ctx, g=g, indptr=indptr.numpy(), indices=indices.numpy(), feat=feat.numpy(),
                seeds=seeds, ws=ws, wn=wn, bs=bs)


@pytest.fixture(scope="module", params=["medium", "large"])
def big(request):
    return _setup(request.param)


def _run_batches(e, cache, batches):
    dci, gu, w, ctx, g = e["dci"], e["gu"], e["w"], e["ctx"], e["g"]
    blk = dci.Blocks(ctx, w.num_nodes, w.batch_size, w.fanouts)
    x = torch.empty(blk.cap_nodes[-1], w.feat_dim, dtype=torch.float32, device="cuda")
    logits = torch.empty(w.batch_size, w.classes, dtype=torch.float32, device="cuda")
    ws, wn, bs = ([gu.dev(a) for a in e[k]] for k in ("ws", "wn", "bs"))
    seeds_dev = gu.dev(e["seeds"])
    for b in batches:
        sl = slice(b * w.batch_size, min(w.num_seeds, (b + 1) * w.batch_size))
        n_seeds = sl.stop - sl.start
        stats = gu.new_stats()
        dci.dci_sample_khop(ctx, g, cache, seeds_dev[sl], b, w.fanouts, w.rng_seed, blk, stats)
        dci.dci_gather_features(ctx, g, cache, blk.nodes, blk.cap_nodes[-1], x, n_dev=blk.n_input_dev(), stats=stats)
        dci.dci_sage_forward(ctx, blk, x, ws, wn, bs, logits)
        got = gu.blocks_to_host(ctx, blk)
        want = oracle.sample_khop(e["indptr"], e["indices"], e["seeds"][sl], b, w.fanouts, w.rng_seed)
        gu.assert_blocks_equal(got, want)
        n_in = got["n_nodes"][-1]
        want_x = oracle.gather(e["feat"], want.nodes)
        assert x[:n_in].cpu().numpy().tobytes() == want_x.tobytes()
        ref = oracle.sage_forward(want, want_x, e["ws"], e["wn"], e["bs"])
        err = float(np.abs(logits[:n_seeds].cpu().numpy() - ref).max())
        assert err <= 1e-4 * max(1.0, float(np.abs(ref).max())), err
        yield b, want, gu.stats_dict(ctx, stats)


def test_presample_fill_and_batches(big):
    e = big
    dci, gu, w, ctx, g = e["dci"], e["gu"], e["w"], e["ctx"], e["g"]
    # pre-sampling counters, in full
    fc_w, ac_w, _, (edges, nodes) = oracle.presample_count(e["indptr"], e["indices"], e["seeds"], w.batch_size,
                                                          w.n_presample, w.fanouts, w.rng_seed,
                                                          w.presample_first_batch, with_edge_count=False)
    fc = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
    ac = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
    stats = gu.new_stats()
    dci.dci_presample_count(ctx, g, None, gu.dev(e["seeds"]), w.batch_size, 0, w.n_presample,
                            w.presample_first_batch, w.fanouts, w.rng_seed, fc, ac, stats=stats)
    st = gu.stats_dict(ctx, stats)
    assert np.array_equal(fc.cpu().numpy().view(np.uint32), fc_w)
    assert np.array_equal(ac.cpu().numpy().view(np.uint32), ac_w)
    assert (st["edges_sampled"], st["input_nodes"]) == (edges, nodes)

    # the configured budget covers the whole dataset: everything is cached, every access hits
    cache = dci.dci_fill_caches(ctx, g, fc, ac, w.budget_bytes, 3, 7, 0)
    assert (cache.adj_nodes, cache.adj_edges, cache.feat_rows) == (w.num_nodes, w.num_edges, w.num_nodes)
    assert np.array_equal(cache.adj_remap.cpu().numpy(), np.arange(w.num_nodes, dtype=np.int32))
    fr = cache.feat_remap.cpu().numpy()
    fr_w, _, _ = oracle.fill_feat(fc_w, None, cache.cap_feat_bytes, 0, feat_dim=w.feat_dim)
    assert np.array_equal(fr, fr_w)
    for b, want, st in _run_batches(e, cache, [0, w.num_batches - 1]):
        assert st["adj_edge_misses"] == 0 and st["feat_misses"] == 0 and st["feat_hits"] == len(want.nodes)
    del cache

    # a budget under pressure (0.4 GB, the point of the paper's Fig. 11): both caches partial
    budget = 400_000_000
    for policy in (0, 1):
        C_adj, C_feat = oracle.split(budget, 3, 7, w.num_nodes, w.num_edges, w.feat_dim)
        adj_remap, cp, ci = oracle.fill_adj(e["indptr"], e["indices"], ac_w, C_adj)
        feat_remap, _, k = oracle.fill_feat(fc_w, None, C_feat, policy, feat_dim=w.feat_dim)
        cache = dci.dci_fill_caches(ctx, g, fc, ac, budget, 3, 7, policy)
        assert (cache.cap_adj_bytes, cache.cap_feat_bytes) == (C_adj, C_feat)
        assert (cache.adj_nodes, cache.adj_edges, cache.feat_rows) == (len(cp) - 1, len(ci), k)
        assert 0 < cache.adj_nodes < w.num_nodes and 0 < k < w.num_nodes
        assert np.array_equal(cache.adj_remap.cpu().numpy(), adj_remap)
        assert np.array_equal(cache.feat_remap.cpu().numpy(), feat_remap)
        base = cache.buf.data_ptr()

        def view(addr, n, dtype):
            off = addr - base
            return cache.buf[off:off + n * torch.tensor([], dtype=dtype).element_size()].view(dtype)

        assert np.array_equal(view(cache.c.c_indptr, len(cp), torch.int64).cpu().numpy(), cp)
        assert np.array_equal(view(cache.c.c_indices, len(ci), torch.int64).cpu().numpy(), ci)
        rows = np.flatnonzero(feat_remap >= 0)
        pick = rows[np.random.default_rng(policy).permutation(len(rows))[:20000]]
        got_rows = view(cache.c.feat_cache, k * w.feat_dim, torch.float32).view(k, w.feat_dim)[
            torch.from_numpy(feat_remap[pick].astype(np.int64)).cuda()].cpu().numpy()
        assert got_rows.tobytes() == e["feat"][pick].tobytes()
        if policy == 0:
            for b, want, st in _run_batches(e, cache, [1]):
                hit = feat_remap[want.nodes] >= 0
                assert (st["feat_hits"], st["feat_misses"]) == (int(hit.sum()), int((~hit).sum()))
                assert st["feat_hits"] > 0 and st["feat_misses"] > 0
                assert st["adj_edge_hits"] > 0 and st["adj_edge_misses"] > 0
        del cache


def test_batches_in_flight_full_size(big):
    """dci_infer_batches at full size, the launch configuration of bench.py's pipelined region: six consecutive
    batches on four lanes through partially filled caches (0.4 GB), every batch's logits against the oracle and the
    blocks / gathered rows of the batch each lane ran last, bit for bit."""
    e = big
    dci, gu, w, ctx, g = e["dci"], e["gu"], e["w"], e["ctx"], e["g"]
    fc = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
    ac = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
    seeds_dev = gu.dev(e["seeds"])
    dci.dci_presample_count(ctx, g, None, seeds_dev, w.batch_size, 0, w.n_presample, w.presample_first_batch,
                            w.fanouts, w.rng_seed, fc, ac)
    cache = dci.dci_fill_caches(ctx, g, fc, ac, 400_000_000, 3, 7, 0)
    assert 0 < cache.adj_nodes < w.num_nodes and 0 < cache.feat_rows < w.num_nodes
    ws, wn, bs = ([gu.dev(a) for a in e[k]] for k in ("ws", "wn", "bs"))
    lanes = [dci.Lane(g, w.batch_size, w.fanouts, w.dims) for _ in range(4)]
    first, count = 2, 6
    logits = torch.full((w.num_seeds, w.classes), float("nan"), dtype=torch.float32, device="cuda")
    stats = gu.new_stats()
    torch.cuda.synchronize()
    dci.dci_infer_batches(lanes, g, cache, seeds_dev, w.batch_size, first, count, w.fanouts, w.rng_seed, 0, ws, wn, bs,
                          logits, stats)
    for ln in lanes:
        ln.ctx.sync()
    out = logits.cpu().numpy()
    edges = 0
    last_of_lane = {k: first + k + 4 * ((count - 1 - k) // 4) for k in range(4)}      # lane k ran first+k, first+k+4, ...
    for b in range(first, first + count):
        sl = slice(b * w.batch_size, (b + 1) * w.batch_size)
        want = oracle.sample_khop(e["indptr"], e["indices"], e["seeds"][sl], b, w.fanouts, w.rng_seed)
        want_x = oracle.gather(e["feat"], want.nodes)
        ref = oracle.sage_forward(want, want_x, e["ws"], e["wn"], e["bs"])
        err = float(np.abs(out[sl] - ref).max())
        assert err <= 1e-4 * max(1.0, float(np.abs(ref).max())), (b, err)
        edges += int(want.n_edges.sum())
        for k, lb in last_of_lane.items():
            if lb == b:
                gu.assert_blocks_equal(gu.blocks_to_host(lanes[k].ctx, lanes[k].blocks), want)
                assert lanes[k].x[:len(want.nodes)].cpu().numpy().tobytes() == want_x.tobytes()
    assert np.isnan(out[:first * w.batch_size]).all() and np.isnan(out[(first + count) * w.batch_size:]).all()
    st = gu.stats_dict(ctx, stats)
    assert st["edges_sampled"] == edges and st["adj_edge_hits"] > 0 and st["adj_edge_misses"] > 0
    assert st["feat_hits"] > 0 and st["feat_misses"] > 0


def test_element_granular_cache_full_size(big):
    """Algorithm 1 as printed, at full size: second-level sort of every counted node's list (in the pinned host
    structure too), a last node cached in part, blocks bit for bit and hits counted per position.  The host lists
    are restored afterwards."""
    e = big
    dci, gu, w, ctx, g = e["dci"], e["gu"], e["w"], e["ctx"], e["g"]
    original = e["indices"].copy()
    try:
        fc_w, ac_w, ec_w, _ = oracle.presample_count(e["indptr"], e["indices"], e["seeds"], w.batch_size, w.n_presample,
                                                     w.fanouts, w.rng_seed, w.presample_first_batch, with_edge_count=True)
        fc = gu.dev(fc_w.view(np.int32))
        ac = gu.dev(ac_w.view(np.int32))
        ec = torch.zeros(w.num_edges, dtype=torch.int32, device="cuda")
        fz = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
        az = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
        dci.dci_presample_count(ctx, g, None, gu.dev(e["seeds"]), w.batch_size, 0, w.n_presample, w.presample_first_batch,
                                w.fanouts, w.rng_seed, fz, az, ec)
        ctx.sync()
        assert np.array_equal(ec.cpu().numpy().view(np.uint32), ec_w)
        budget = 400_000_000
        C_adj, C_feat = oracle.split(budget, 3, 7, w.num_nodes, w.num_edges, w.feat_dim)
        remap, cp, ci, idx, pn, pd = oracle.fill_adj_element(e["indptr"], original, ec_w, C_adj)
        cache = dci.dci_fill_caches(ctx, g, fc, ac, budget, 3, 7, dci.DCI_FILL_ADJ_ELEMENTS, edge_count=ec)
        assert cache.cap_adj_bytes == C_adj
        assert (cache.adj_nodes, cache.adj_edges) == (len(cp) - 1, len(ci))
        assert (cache.adj_partial_node, cache.adj_partial_deg) == (pn, pd) and pn >= 0
        assert np.array_equal(cache.adj_remap.cpu().numpy(), remap)
        assert np.array_equal(e["indices"], idx), "host lists after the fill"
        base = cache.buf.data_ptr()
        view = lambda addr, n: cache.buf[addr - base:addr - base + 8 * n].view(torch.int64).cpu().numpy()
        assert np.array_equal(view(cache.c.c_indptr, len(cp)), cp)
        assert np.array_equal(view(cache.c.c_indices, len(ci)), ci)
        # one batch through the cache, the partial node among its seeds
        b = 1
        seeds = e["seeds"][b * w.batch_size:(b + 1) * w.batch_size].copy()
        seeds[-1] = pn
        want = oracle.sample_khop(e["indptr"], idx, seeds, b, w.fanouts, w.rng_seed)
        hits = host = 0
        for h in range(w.n_hops):
            _, _, c4 = oracle.sample_hop_cached(e["indptr"], idx, remap, cp, ci, want.nodes[:want.n_nodes[h]], b, h,
                                                w.fanouts[h], w.rng_seed, pn, pd)
            hits += int(c4[2]); host += int(c4[3])
        blk = dci.Blocks(ctx, w.num_nodes, w.batch_size, w.fanouts)
        stats = gu.new_stats()
        dci.dci_sample_khop(ctx, g, cache, gu.dev(seeds), b, w.fanouts, w.rng_seed, blk, stats)
        gu.assert_blocks_equal(gu.blocks_to_host(ctx, blk), want)
        st = gu.stats_dict(ctx, stats)
        assert (st["adj_edge_hits"], st["adj_edge_misses"]) == (hits, host) and hits > 0 and host > 0
    finally:
        e["indices"][:] = original


@pytest.fixture(scope="module")
def yelp():
    return _setup("yelp")


def test_table3_model_on_amazon_shape():
    """The sum-aggregate GraphSAGE of Table III on a graph of Amazon's shape (Table II: 1.6 M nodes, 132 M edges,
    200 features, 107 classes): one whole batch through partly filled caches against the oracle."""
    e = _setup("amazon")
    dci, gu, w, ctx, g = e["dci"], e["gu"], e["w"], e["ctx"], e["g"]
    assert w.dims == (200, 128, 128, 107)
    fc = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
    ac = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
    seeds_dev = gu.dev(e["seeds"])
    dci.dci_presample_count(ctx, g, None, seeds_dev, w.batch_size, 0, w.n_presample, w.presample_first_batch, w.fanouts,
                            w.rng_seed, fc, ac)
    cache = dci.dci_fill_caches(ctx, g, fc, ac, 600_000_000, 3, 7, 0)
    assert 0 < cache.feat_rows < w.num_nodes and 0 < cache.adj_nodes < w.num_nodes
    blk = dci.Blocks(ctx, w.num_nodes, w.batch_size, w.fanouts)
    x = torch.empty(blk.cap_nodes[-1], w.feat_dim, dtype=torch.float32, device="cuda")
    logits = torch.empty(w.batch_size, w.classes, dtype=torch.float32, device="cuda")
    ws, wn, bs = ([gu.dev(a) for a in e[k]] for k in ("ws", "wn", "bs"))
    b = 2
    sl = slice(b * w.batch_size, (b + 1) * w.batch_size)
    dci.dci_sample_khop(ctx, g, cache, seeds_dev[sl], b, w.fanouts, w.rng_seed, blk)
    dci.dci_gather_forward(ctx, g, cache, blk, x, 1, ws, wn, bs, logits)
    got = gu.blocks_to_host(ctx, blk)
    want = oracle.sample_khop(e["indptr"], e["indices"], e["seeds"][sl], b, w.fanouts, w.rng_seed)
    gu.assert_blocks_equal(got, want)
    ref = oracle.gnn_forward(1, want, oracle.gather(e["feat"], want.nodes), e["ws"], e["wn"], e["bs"])
    err = float(np.abs(logits.cpu().numpy() - ref).max())
    assert err <= 1e-4 * max(1.0, float(np.abs(ref).max())), err


@pytest.mark.parametrize("model", [1, 2])
def test_table3_models_on_yelp_shape(yelp, model):
    """The three-layer, hidden-128 sum-aggregate GraphSAGE and averaging GCN (Table III) on a graph of Yelp's shape
    (Table II): one whole batch, dual cache filled, logits against the fp64 oracle."""
    e = yelp
    dci, gu, w, ctx, g = e["dci"], e["gu"], e["w"], e["ctx"], e["g"]
    assert w.dims == (300, 128, 128, 100)
    fc = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
    ac = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
    seeds_dev = gu.dev(e["seeds"])
    dci.dci_presample_count(ctx, g, None, seeds_dev, w.batch_size, 0, w.n_presample, w.presample_first_batch, w.fanouts,
                            w.rng_seed, fc, ac)
    cache = dci.dci_fill_caches(ctx, g, fc, ac, 200_000_000, 3, 7, 0)
    assert 0 < cache.feat_rows < w.num_nodes
    blk = dci.Blocks(ctx, w.num_nodes, w.batch_size, w.fanouts)
    x = torch.empty(blk.cap_nodes[-1], w.feat_dim, dtype=torch.float32, device="cuda")
    logits = torch.empty(w.batch_size, w.classes, dtype=torch.float32, device="cuda")
    ws, wn, bs = ([gu.dev(a) for a in e[k]] for k in ("ws", "wn", "bs"))
    b = 3
    sl = slice(b * w.batch_size, (b + 1) * w.batch_size)
    dci.dci_sample_khop(ctx, g, cache, seeds_dev[sl], b, w.fanouts, w.rng_seed, blk)
    dci.dci_gather_features(ctx, g, cache, blk.nodes, blk.cap_nodes[-1], x, n_dev=blk.n_input_dev())
    dci.dci_gnn_forward(ctx, blk, x, model, None if model == 2 else ws, wn, bs, logits)
    want = oracle.sample_khop(e["indptr"], e["indices"], e["seeds"][sl], b, w.fanouts, w.rng_seed)
    gu.assert_blocks_equal(gu.blocks_to_host(ctx, blk), want)
    want_x = oracle.gather(e["feat"], want.nodes)
    assert x[:len(want.nodes)].cpu().numpy().tobytes() == want_x.tobytes()
    ref = oracle.gnn_forward(model, want, want_x, e["ws"], e["wn"], e["bs"])
    err = float(np.abs(logits.cpu().numpy() - ref).max())
    assert err <= 1e-4 * max(1.0, float(np.abs(ref).max())), err
