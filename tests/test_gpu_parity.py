"""GPU parity: every call of the C boundary against the CPU oracle on the same seeded inputs.
Integer outputs (blocks, counters, remaps, cache arrays, gathered rows) are compared bit for
bit; logits within 1e-4 of the largest oracle logit of the batch."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env(tiny):
    import paper_2503_01281_amd as dci
    from tests import gpu_util
    assert torch.cuda.is_available(), "these tests need the GPU"
    ctx = dci.Context(0)
    g = gpu_util.make_graph(tiny["indptr"], tiny["indices"], tiny["feat"])
    return dict(dci=dci, gu=gpu_util, ctx=ctx, graph=g, tiny=tiny, w=tiny["w"])


def _oracle_caches(tiny, w, ts=3, tf=7, policy=0, budget=None, spill=True):
    fc, ac, _, _ = oracle.presample_count(tiny["indptr"], tiny["indices"], tiny["seeds"], w.batch_size,
                                          w.n_presample, w.fanouts, w.rng_seed, w.presample_first_batch,
                                          with_edge_count=False)
    C_adj, C_feat = oracle.split(w.budget_bytes if budget is None else budget, ts, tf, w.num_nodes, w.num_edges,
                                 w.feat_dim, spill)
    adj_remap, cp, ci = oracle.fill_adj(tiny["indptr"], tiny["indices"], ac, C_adj)
    feat_remap, fcache, k = oracle.fill_feat(fc, tiny["feat"], C_feat, policy)
    return dict(fc=fc, ac=ac, C_adj=C_adj, C_feat=C_feat, adj_remap=adj_remap, c_indptr=cp, c_indices=ci,
                feat_remap=feat_remap, feat_cache=fcache, k=k)


def test_sample_all_batches_no_cache(env):
    dci, gu, ctx, g, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "graph", "tiny", "w"))
    seeds_dev = gu.dev(tiny["seeds"])
    blk = dci.Blocks(ctx, w.num_nodes, w.batch_size, w.fanouts)
    stats = gu.new_stats()
    edges = nodes = 0
    for b in range(w.num_batches):
        s = seeds_dev[b * w.batch_size:(b + 1) * w.batch_size]
        dci.dci_sample_khop(ctx, g, None, s, b, w.fanouts, w.rng_seed, blk, stats)
        got = gu.blocks_to_host(ctx, blk)
        want = oracle.sample_khop(tiny["indptr"], tiny["indices"], tiny["seeds"][b * w.batch_size:(b + 1) * w.batch_size],
                                  b, w.fanouts, w.rng_seed)
        gu.assert_blocks_equal(got, want)
        edges += int(want.n_edges.sum())
        nodes += int(want.n_nodes[-1])
    st = gu.stats_dict(ctx, stats)
    assert st["edges_sampled"] == edges and st["input_nodes"] == nodes
    assert st["adj_edge_misses"] == edges and st["adj_edge_hits"] == 0 and st["adj_node_hits"] == 0


def test_sample_with_cache_is_transparent_and_counts_hits(env):
    dci, gu, ctx, g, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "graph", "tiny", "w"))
    oc = _oracle_caches(tiny, w)
    cache = gu.upload_cache(oc["adj_remap"], oc["c_indptr"], oc["c_indices"], oc["feat_remap"], oc["feat_cache"])
    blk = dci.Blocks(ctx, w.num_nodes, w.batch_size, w.fanouts)
    for b in (0, 3, 7):
        seeds = tiny["seeds"][b * w.batch_size:(b + 1) * w.batch_size]
        stats = gu.new_stats()
        dci.dci_sample_khop(ctx, g, cache, gu.dev(seeds), b, w.fanouts, w.rng_seed, blk, stats)
        got = gu.blocks_to_host(ctx, blk)
        want = oracle.sample_khop(tiny["indptr"], tiny["indices"], seeds, b, w.fanouts, w.rng_seed)
        gu.assert_blocks_equal(got, want)
        nh = nm = eh = em = 0
        for h in range(w.n_hops):
            frontier = want.nodes[:want.n_nodes[h]]
            hit = oc["adj_remap"][frontier] >= 0
            rows = np.diff(want.blk_indptr[h])
            nh += int(hit.sum()); nm += int((~hit).sum()); eh += int(rows[hit].sum()); em += int(rows[~hit].sum())
        st = gu.stats_dict(ctx, stats)
        assert (st["adj_node_hits"], st["adj_node_misses"], st["adj_edge_hits"], st["adj_edge_misses"]) == (nh, nm, eh, em)
        assert nh > 0 and nm > 0


@pytest.mark.parametrize("fanouts", [(3,), (8, 8), (16, 2), (9, 17), (25, 10), (33,), (64,), (40, 3), (1, 1, 1, 1),
                                     (2, 2, 2, 2, 2, 2, 2, 2)])
@pytest.mark.parametrize("n_seeds", [1, 7, 300])
def test_sample_fanout_and_batch_shapes(env, fanouts, n_seeds):
    dci, gu, ctx, g, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "graph", "tiny", "w"))
    seeds = tiny["seeds"][100:100 + n_seeds]
    blk = dci.Blocks(ctx, w.num_nodes, n_seeds, fanouts)
    dci.dci_sample_khop(ctx, g, None, gu.dev(seeds), 17, fanouts, 99, blk)
    got = gu.blocks_to_host(ctx, blk)
    want = oracle.sample_khop(tiny["indptr"], tiny["indices"], seeds, 17, fanouts, 99)
    gu.assert_blocks_equal(got, want)


def test_sample_degenerate_inputs(env, small_graphs):
    dci, gu, ctx = env["dci"], env["gu"], env["ctx"]
    indptr, indices = small_graphs[3]          # isolated nodes, a self loop, a duplicated edge
    g = gu.make_graph(indptr, indices, None)
    for seeds in ([], [0, 4], [1], [1, 1, 3], [0, 1, 2, 3, 4]):
        seeds = np.array(seeds, dtype=np.int64)
        blk = dci.Blocks(ctx, 5, len(seeds), (3, 2))
        sd = gu.dev(seeds) if len(seeds) else torch.zeros(1, dtype=torch.int64, device="cuda")[:0]
        dci.dci_sample_khop(ctx, g, None, sd, 0, (3, 2), 4, blk)
        got = gu.blocks_to_host(ctx, blk)
        want = oracle.sample_khop(indptr, indices, seeds, 0, (3, 2), 4)
        gu.assert_blocks_equal(got, want)


def test_sample_rejects_bad_arguments(env):
    dci, gu, ctx, g, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "graph", "tiny", "w"))
    seeds = gu.dev(tiny["seeds"][:16])
    blk = dci.Blocks(ctx, w.num_nodes, 16, (5, 10))
    with pytest.raises(dci.DciError) as e:
        dci.dci_sample_khop(ctx, g, None, seeds, 0, (5, 65), 4, blk)
    assert e.value.code == -1
    with pytest.raises(dci.DciError) as e:
        dci.dci_sample_khop(ctx, g, None, seeds, 1 << 32, (5, 10), 4, blk)
    assert e.value.code == -1
    small = dci.Blocks(ctx, w.num_nodes, 4, (5, 10))
    with pytest.raises(dci.DciError) as e:
        dci.dci_sample_khop(ctx, g, None, seeds, 0, (5, 10), 4, small)
    assert e.value.code == -2 and "needed" in str(e.value)
    # the sizes the refused call needed are there to be read
    cn, ce, ws_need = ctx.last_required()
    want_n, want_e = dci.blocks_bounds(w.num_nodes, 16, (5, 10))
    assert cn[:3] == want_n and ce[:2] == want_e and cn[3:] == [0] * 6 and ce[2:] == [0] * 6 and ws_need > 0


@pytest.mark.parametrize("F", [64, 100, 602, 63, 1, 256])
def test_gather_hit_and_miss_paths(env, F):
    dci, gu, ctx = env["dci"], env["gu"], env["ctx"]
    N = 3000
    feat = synth.features(N, F, 21)
    rng = np.random.default_rng(F)
    ids = rng.integers(0, N, 5000).astype(np.int64)
    fc = rng.integers(0, 5, N).astype(np.uint32)
    remap, fcache, k = oracle.fill_feat(fc, feat, (N // 3) * 4 * F, 1)
    indptr = np.zeros(N + 1, dtype=np.int64)
    g = gu.make_graph(indptr, np.zeros(1, dtype=np.int64)[:0], feat)
    cache = gu.upload_cache(np.full(N, -1, dtype=np.int32), np.zeros(1, dtype=np.int64), np.zeros(0, dtype=np.int64),
                            remap, fcache)
    want = oracle.gather(feat, ids)
    ids_dev = gu.dev(ids)
    for c in (None, cache):
        out = torch.full((len(ids) + 3, F), -7.0, dtype=torch.float32, device="cuda")
        stats = gu.new_stats()
        dci.dci_gather_features(ctx, g, c, ids_dev, len(ids), out, stats=stats)
        st = gu.stats_dict(ctx, stats)
        assert out[:len(ids)].cpu().numpy().tobytes() == want.tobytes()
        assert (out[len(ids):] == -7.0).all()                       # nothing written past n
        hits = int((remap[ids] >= 0).sum()) if c is not None else 0
        assert (st["feat_hits"], st["feat_misses"]) == (hits, len(ids) - hits)
    # row count taken from device memory
    n_dev = torch.tensor([1234], dtype=torch.int64, device="cuda")
    out = torch.full((len(ids), F), -7.0, dtype=torch.float32, device="cuda")
    dci.dci_gather_features(ctx, g, cache, ids_dev, len(ids), out, n_dev=n_dev.data_ptr())
    ctx.sync()
    assert out[:1234].cpu().numpy().tobytes() == want[:1234].tobytes() and (out[1234:] == -7.0).all()


def test_presample_counts(env):
    dci, gu, ctx, g, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "graph", "tiny", "w"))
    fc_w, ac_w, ec_w, (edges, nodes) = oracle.presample_count(tiny["indptr"], tiny["indices"], tiny["seeds"], w.batch_size,
                                                              w.n_presample, w.fanouts, w.rng_seed,
                                                              w.presample_first_batch)
    seeds = gu.dev(tiny["seeds"])
    fc = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
    ac = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
    ec = torch.zeros(w.num_edges, dtype=torch.int32, device="cuda")
    stats = gu.new_stats()
    # two calls of four batches each must add up to the oracle's eight
    dci.dci_presample_count(ctx, g, None, seeds, w.batch_size, 0, 4, w.presample_first_batch, w.fanouts, w.rng_seed,
                            fc, ac, ec, stats=stats)
    scratch = torch.empty(dci.blocks_bounds(w.num_nodes, w.batch_size, w.fanouts)[0][-1] * w.feat_dim,
                          dtype=torch.float32, device="cuda")
    dci.dci_presample_count(ctx, g, None, seeds, w.batch_size, 4, 4, w.presample_first_batch + 4, w.fanouts,
                            w.rng_seed, fc, ac, ec, feat_scratch=scratch, stats=stats)
    st = gu.stats_dict(ctx, stats)
    assert np.array_equal(fc.cpu().numpy().view(np.uint32), fc_w)
    assert np.array_equal(ac.cpu().numpy().view(np.uint32), ac_w)
    assert np.array_equal(ec.cpu().numpy().view(np.uint32), ec_w)
    assert st["edges_sampled"] == edges and st["input_nodes"] == nodes
    assert st["t_sample_ns"] > 0 and st["t_feature_ns"] > 0


def test_presample_counts_through_caches(env):
    """Counting while the caches are in use: the same counters whether lists come from the host, from a
    node-granular cache or from an element-granular one with a partly cached node (element counters are indexed by
    position in the host list, which the element-granular fill has reordered)."""
    dci, gu, ctx, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "tiny", "w"))
    seeds = gu.dev(tiny["seeds"])
    fc0, ac0, ec0 = _element_counts(tiny, w)
    for elements in (False, True):
        g = gu.make_graph(tiny["indptr"], tiny["indices"].copy(), tiny["feat"])
        flags = dci.DCI_FILL_STRICT_SPLIT | (dci.DCI_FILL_ADJ_ELEMENTS if elements else 0)
        cache = dci.dci_fill_caches(ctx, g, gu.dev(fc0.view(np.int32)), gu.dev(ac0.view(np.int32)), 300_024 + 400_000, 3, 4,
                                    flags, edge_count=gu.dev(ec0.view(np.int32)))
        ctx.sync()
        assert 0 < cache.adj_nodes < w.num_nodes and 0 < cache.feat_rows < w.num_nodes
        assert (cache.adj_partial_node >= 0) == elements
        host_lists = g.indices.numpy().copy()
        fc_w, ac_w, ec_w, (edges, nodes) = oracle.presample_count(tiny["indptr"], host_lists, tiny["seeds"], w.batch_size,
                                                                  4, w.fanouts, w.rng_seed, 77)
        fc = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
        ac = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
        ec = torch.zeros(w.num_edges, dtype=torch.int32, device="cuda")
        stats = gu.new_stats()
        scratch = torch.empty(dci.blocks_bounds(w.num_nodes, w.batch_size, w.fanouts)[0][-1] * w.feat_dim,
                              dtype=torch.float32, device="cuda")
        dci.dci_presample_count(ctx, g, cache, seeds, w.batch_size, 0, 4, 77, w.fanouts, w.rng_seed, fc, ac, ec,
                                feat_scratch=scratch, stats=stats)
        st = gu.stats_dict(ctx, stats)
        assert np.array_equal(fc.cpu().numpy().view(np.uint32), fc_w)
        assert np.array_equal(ac.cpu().numpy().view(np.uint32), ac_w)
        assert np.array_equal(ec.cpu().numpy().view(np.uint32), ec_w)
        assert st["edges_sampled"] == edges and st["input_nodes"] == nodes
        assert st["adj_edge_hits"] > 0 and st["adj_edge_misses"] > 0 and st["feat_hits"] > 0 and st["feat_misses"] > 0
        assert st["adj_edge_hits"] + st["adj_edge_misses"] == edges


def _check_fill(env, budget, ts, tf, policy, spill=True):
    dci, gu, ctx, g, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "graph", "tiny", "w"))
    oc = _oracle_caches(tiny, w, ts, tf, policy, budget, spill)
    cache = dci.dci_fill_caches(ctx, g, gu.dev(oc["fc"].view(np.int32)), gu.dev(oc["ac"].view(np.int32)), budget, ts, tf,
                                policy | (0 if spill else 0x100))
    K, M, k = cache.adj_nodes, cache.adj_edges, cache.feat_rows
    assert (cache.cap_adj_bytes, cache.cap_feat_bytes) == (oc["C_adj"], oc["C_feat"])
    assert (K, M, k) == (len(oc["c_indptr"]) - 1, len(oc["c_indices"]), oc["k"])
    assert np.array_equal(cache.adj_remap.cpu().numpy(), oc["adj_remap"])
    assert np.array_equal(cache.feat_remap.cpu().numpy(), oc["feat_remap"])
    assert cache.adj_bytes <= max(oc["C_adj"], 8) and cache.feat_bytes <= oc["C_feat"]
    base = cache.buf.data_ptr() + cache.buf_offset

    def view(addr, n, dtype):
        off = addr - cache.buf.data_ptr()
        nbytes = n * torch.tensor([], dtype=dtype).element_size()
        return cache.buf[off:off + nbytes].view(dtype).cpu().numpy()

    assert cache.c.feat_cache == base or k == 0
    if k:
        assert view(cache.c.feat_cache, k * w.feat_dim, torch.float32).tobytes() == oc["feat_cache"].tobytes()
    if K:
        assert np.array_equal(view(cache.c.c_indptr, K + 1, torch.int64), oc["c_indptr"])
    if M:
        assert np.array_equal(view(cache.c.c_indices, M, torch.int64), oc["c_indices"])
    return cache


@pytest.mark.parametrize("policy", [0, 1])
@pytest.mark.parametrize("budget,ts,tf", [(1_127_220, 3, 7), (1_127_220, 7, 3), (1_127_220, 1, 0), (1_127_220, 0, 1),
                                          (5_636_104, 3, 7), (5_636_103, 1, 1), (20, 1, 1), (0, 1, 1),
                                          (300_001, 0, 0), (3_000_000, 9, 1), (3_000_000, 1, 9)])
def test_fill_caches_matches_oracle(env, budget, ts, tf, policy):
    _check_fill(env, budget, ts, tf, policy)


def _element_counts(tiny, w):
    _, ac, ec, _ = oracle.presample_count(tiny["indptr"], tiny["indices"], tiny["seeds"], w.batch_size, w.n_presample,
                                          w.fanouts, w.rng_seed, w.presample_first_batch, with_edge_count=True)
    fc = np.zeros(w.num_nodes, dtype=np.uint32)
    return fc, ac, ec


@pytest.mark.parametrize("c_adj", [0, 8, 24, 40_000, 300_000, 300_008, 300_016, 300_024, 900_001, 1_441_799, 1_441_800])
def test_element_granular_fill_matches_oracle(env, c_adj):
    """Algorithm 1 as printed: second-level sort inside the nodes (applied to the host lists as well) and a last
    node cached in part.  Strict split with t_feature = 0 hands the whole budget to the adjacency cache."""
    dci, gu, ctx, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "tiny", "w"))
    fc, ac, ec = _element_counts(tiny, w)
    g = gu.make_graph(tiny["indptr"], tiny["indices"].copy(), tiny["feat"])      # the fill rewrites the lists
    want = oracle.fill_adj_element(tiny["indptr"], tiny["indices"], ec, c_adj)
    remap, cp, ci, idx, pn, pd = want
    cache = dci.dci_fill_caches(ctx, g, gu.dev(fc.view(np.int32)), gu.dev(ac.view(np.int32)), c_adj, 1, 0,
                                dci.DCI_FILL_STRICT_SPLIT | dci.DCI_FILL_ADJ_ELEMENTS, edge_count=gu.dev(ec.view(np.int32)))
    ctx.sync()
    assert cache.cap_adj_bytes == c_adj and cache.feat_rows == 0
    assert (cache.adj_nodes, cache.adj_edges) == (len(cp) - 1, len(ci))
    assert (cache.adj_partial_node, cache.adj_partial_deg) == (pn, pd)
    assert np.array_equal(cache.adj_remap.cpu().numpy(), remap)
    assert np.array_equal(g.indices.numpy(), idx), "host lists after the fill"

    def view(addr, n):
        off = addr - cache.buf.data_ptr()
        return cache.buf[off:off + 8 * n].view(torch.int64).cpu().numpy()

    if cache.adj_nodes:
        assert np.array_equal(view(cache.c.c_indptr, cache.adj_nodes + 1), cp)
    if cache.adj_edges:
        assert np.array_equal(view(cache.c.c_indices, cache.adj_edges), ci)
    if c_adj in (300_016, 300_024):
        assert pn >= 0


def test_element_granular_fill_on_small_graphs_with_random_counts(env, small_graphs):
    """Small graphs (isolated nodes, a self loop, duplicate edges), random element counts with many zeros and ties,
    budgets from nothing to everything: remap, cache arrays, the partly cached node and the rewritten host lists."""
    dci, gu, ctx = env["dci"], env["gu"], env["ctx"]
    rng = np.random.default_rng(31)
    for indptr, indices in small_graphs:
        n, e = len(indptr) - 1, len(indices)
        feat = np.zeros((n, 4), dtype=np.float32)
        whole = (n + 1 + e) * 8
        for trial in range(5):
            ec = (rng.integers(0, 5, e) * rng.integers(0, 2, e)).astype(np.uint32)
            ac = np.add.reduceat(np.concatenate([ec, [0]]).astype(np.uint64), indptr[:-1])[:n] if e else np.zeros(n, np.uint64)
            ac = np.where(np.diff(indptr) > 0, ac, 0).astype(np.uint32)
            for c_adj in [0, 16, 40, int(rng.integers(16, whole)), int(rng.integers(16, whole)), whole - 1, whole]:
                g = gu.make_graph(indptr, indices.copy(), feat)
                remap, cp, ci, idx, pn, pd = oracle.fill_adj_element(indptr, indices, ec, c_adj)
                cache = dci.dci_fill_caches(ctx, g, gu.dev(np.zeros(n, np.int32)), gu.dev(ac.view(np.int32)), c_adj, 1, 0,
                                            dci.DCI_FILL_STRICT_SPLIT | dci.DCI_FILL_ADJ_ELEMENTS,
                                            edge_count=gu.dev(ec.view(np.int32)) if e else torch.zeros(1, dtype=torch.int32, device="cuda"))
                ctx.sync()
                what = f"n={n} e={e} trial={trial} c_adj={c_adj}"
                assert (cache.adj_nodes, cache.adj_edges) == (len(cp) - 1, len(ci)), what
                assert (cache.adj_partial_node, cache.adj_partial_deg) == (pn, pd), what
                assert np.array_equal(cache.adj_remap.cpu().numpy(), remap), what
                assert np.array_equal(g.indices.numpy(), idx), what
                view = lambda addr, k: cache.buf[addr - cache.buf.data_ptr():addr - cache.buf.data_ptr() + 8 * k].view(torch.int64).cpu().numpy()
                if cache.adj_nodes:
                    assert np.array_equal(view(cache.c.c_indptr, cache.adj_nodes + 1), cp), what
                if cache.adj_edges:
                    assert np.array_equal(view(cache.c.c_indices, cache.adj_edges), ci), what


def test_element_granular_cache_is_transparent_and_counts_hits_per_position(env):
    dci, gu, ctx, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "tiny", "w"))
    fc, ac, ec = _element_counts(tiny, w)
    g = gu.make_graph(tiny["indptr"], tiny["indices"].copy(), tiny["feat"])
    c_adj = 300_024
    remap, cp, ci, idx, pn, pd = oracle.fill_adj_element(tiny["indptr"], tiny["indices"], ec, c_adj)
    assert pn >= 0
    cache = dci.dci_fill_caches(ctx, g, gu.dev(fc.view(np.int32)), gu.dev(ac.view(np.int32)), c_adj, 1, 0,
                                dci.DCI_FILL_STRICT_SPLIT | dci.DCI_FILL_ADJ_ELEMENTS, edge_count=gu.dev(ec.view(np.int32)))
    uploaded = gu.upload_cache(remap, cp, ci, np.full(w.num_nodes, -1), np.zeros((0, w.feat_dim), np.float32), pn, pd)
    seeds = np.concatenate([tiny["seeds"][512:767], [pn]])
    want = oracle.sample_khop(tiny["indptr"], idx, seeds, 2, w.fanouts, w.rng_seed)
    hits = host = 0
    for h in range(w.n_hops):
        _, _, c4 = oracle.sample_hop_cached(tiny["indptr"], idx, remap, cp, ci, want.nodes[:want.n_nodes[h]], 2, h,
                                            w.fanouts[h], w.rng_seed, pn, pd)
        hits += int(c4[2]); host += int(c4[3])
    assert host > 0
    # host lines: a missed node costs the lines of its two list bounds and of the ids it reads; the node cached in
    # part costs one line of bounds (where its host list starts) and the lines of the ids beyond its cached length
    blines = ilines = slot_rows = all_rows = 0
    for h in range(w.n_hops):
        frontier = want.nodes[:want.n_nodes[h]]
        bi = want.blk_indptr[h]
        for i, v in enumerate(frontier):
            v = int(v)
            r = int(remap[v])
            pos = want.src_pos[h][bi[i]:bi[i + 1]]
            all_rows += 1
            if r < 0:
                if h == 0 or i >= int(want.n_nodes[h - 1]):   # fetched once per batch, noted for the later hops
                    blines += _host_lines(g.indptr.data_ptr(), [8 * v, 8 * (v + 1)])
            else:
                slot_rows += 1
                pos = pos[pos >= int(cp[r + 1] - cp[r])]
                blines += 1 if len(pos) else 0
            if len(pos):
                ilines += _host_lines(g.indices.data_ptr(), 8 * (int(tiny["indptr"][v]) + pos))
    for c_ in (cache, uploaded):
        blk = dci.Blocks(ctx, w.num_nodes, len(seeds), w.fanouts)
        stats = gu.new_stats()
        dci.dci_sample_khop(ctx, g, c_, gu.dev(seeds), 2, w.fanouts, w.rng_seed, blk, stats)
        gu.assert_blocks_equal(gu.blocks_to_host(ctx, blk), want)
        st = gu.stats_dict(ctx, stats)
        assert (st["adj_edge_hits"], st["adj_edge_misses"]) == (hits, host)
        assert (st["bytes_hbm"], st["bytes_host"]) == (16 * slot_rows + 8 * hits, 16 * (all_rows - slot_rows) + 8 * host)
        assert (st["lines_bounds"], st["lines_ids"]) == (blines, ilines)
    # and the same blocks without any cache, from the reordered host lists alone
    blk = dci.Blocks(ctx, w.num_nodes, len(seeds), w.fanouts)
    dci.dci_sample_khop(ctx, g, None, gu.dev(seeds), 2, w.fanouts, w.rng_seed, blk)
    gu.assert_blocks_equal(gu.blocks_to_host(ctx, blk), want)


def test_element_granular_fill_needs_edge_counts(env):
    dci, gu, ctx, g, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "graph", "tiny", "w"))
    z = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
    with pytest.raises(dci.DciError):
        dci.dci_fill_caches(ctx, g, z, z, 1000, 1, 1, dci.DCI_FILL_ADJ_ELEMENTS)
    # ... and the caller's word that the graph's lists may be rewritten: indices_rw must be graph.indices itself
    ec = torch.zeros(w.num_edges, dtype=torch.int32, device="cuda")
    other = torch.zeros(w.num_edges, dtype=torch.int64, device="cuda")
    with pytest.raises(dci.DciError) as e:
        dci.dci_fill_caches(ctx, g, z, z, 1000, 1, 1, dci.DCI_FILL_ADJ_ELEMENTS, edge_count=ec, indices_rw=other)
    assert e.value.code == -1 and "indices_rw" in str(e.value)


def test_same_call_twice_gives_the_same_bytes(env):
    """Determinism: sampling, gathering and the forward pass of one batch, run twice on one context and once on
    a second context with another stream, leave byte-identical outputs (the float sums run in a fixed order)."""
    dci, gu, g, tiny, w = (env[k] for k in ("dci", "gu", "graph", "tiny", "w"))
    oc = _oracle_caches(tiny, w)
    cache = gu.upload_cache(oc["adj_remap"], oc["c_indptr"], oc["c_indices"], oc["feat_remap"], oc["feat_cache"])
    ws, wn, bs = ([gu.dev(a) for a in tiny[k]] for k in ("w_self", "w_neigh", "bias"))
    seeds = gu.dev(tiny["seeds"][256:512])
    outs = []
    for ctx in (env["ctx"], env["ctx"], dci.Context(0, stream=torch.cuda.Stream())):
        blk = dci.Blocks(ctx, w.num_nodes, w.batch_size, w.fanouts)
        x = torch.zeros(blk.cap_nodes[-1], w.feat_dim, dtype=torch.float32, device="cuda")
        logits = torch.zeros(w.batch_size, w.classes, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        dci.dci_sample_khop(ctx, g, cache, seeds, 1, w.fanouts, w.rng_seed, blk)
        dci.dci_gather_features(ctx, g, cache, blk.nodes, blk.cap_nodes[-1], x, n_dev=blk.n_input_dev())
        dci.dci_sage_forward(ctx, blk, x, ws, wn, bs, logits)
        got = gu.blocks_to_host(ctx, blk)
        outs.append(b"".join([got["nodes"].tobytes()] + [a.tobytes() for a in got["blk_indptr"] + got["blk_src"]]
                             + [x.cpu().numpy().tobytes(), logits.cpu().numpy().tobytes()]))
    assert outs[0] == outs[1] == outs[2]


@pytest.mark.parametrize("budget,ts,tf", [(5_636_104, 9, 1), (5_000_000, 1, 9), (3_000_000, 0, 1), (3_000_000, 1, 0)])
def test_fill_strict_split_and_single_cache(env, budget, ts, tf):
    """Eq. (1) without spill-over; t_sample = 0 gives the single-cache system (no adjacency cache)."""
    cache = _check_fill(env, budget, ts, tf, 0, spill=False)
    if ts == 0:
        assert cache.adj_nodes == 0 and (cache.adj_remap == -1).all()
    if tf == 0:
        assert cache.feat_rows == 0 and (cache.feat_remap == -1).all()


def test_fill_with_many_distinct_counts(env):
    """Counts above 255 exercise more than one radix pass."""
    dci, gu, ctx, g, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "graph", "tiny", "w"))
    rng = np.random.default_rng(3)
    fc = rng.integers(0, 70000, w.num_nodes).astype(np.uint32)
    ac = (rng.integers(0, 3, w.num_nodes) * rng.integers(0, 1 << 20, w.num_nodes)).astype(np.uint32)
    for policy in (0, 1):
        C_adj, C_feat = oracle.split(900_000, 1, 1, w.num_nodes, w.num_edges, w.feat_dim)
        adj_remap, cp, ci = oracle.fill_adj(tiny["indptr"], tiny["indices"], ac, C_adj)
        feat_remap, fcache, k = oracle.fill_feat(fc, tiny["feat"], C_feat, policy)
        cache = dci.dci_fill_caches(ctx, g, gu.dev(fc.view(np.int32)), gu.dev(ac.view(np.int32)), 900_000, 1, 1, policy)
        assert np.array_equal(cache.adj_remap.cpu().numpy(), adj_remap)
        assert np.array_equal(cache.feat_remap.cpu().numpy(), feat_remap)
        assert (cache.adj_nodes, cache.adj_edges, cache.feat_rows) == (len(cp) - 1, len(ci), k)


def _logit_check(got, want):
    tol = 1e-4 * max(1.0, float(np.abs(want).max()))
    err = float(np.abs(got.astype(np.float64) - want).max())
    assert err <= tol, f"max |gpu - oracle| = {err} > {tol}"


@pytest.mark.parametrize("dims,fanouts,n_seeds", [((64, 64, 16), (5, 10), 256), ((602, 256, 41), (3, 4), 70),
                                                  ((100, 256, 256, 47), (2, 3, 4), 33), ((63, 5), (7,), 129),
                                                  ((128, 130, 172), (5, 5), 200), ((256, 256, 64), (10, 25), 40)])
def test_sage_forward_matches_oracle(env, dims, fanouts, n_seeds):
    dci, gu, ctx, g, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "graph", "tiny", "w"))
    seeds = tiny["seeds"][:n_seeds]
    want_blk = oracle.sample_khop(tiny["indptr"], tiny["indices"], seeds, 1, fanouts, 4)
    blk = dci.Blocks(ctx, w.num_nodes, n_seeds, fanouts)
    dci.dci_sample_khop(ctx, g, None, gu.dev(seeds), 1, fanouts, 4, blk)
    feat = synth.features(w.num_nodes, dims[0], 31)
    ws, wn, bs = synth.sage_weights(dims, 32)
    x = feat[want_blk.nodes]
    want = oracle.sage_forward(want_blk, x, ws, wn, bs)
    x_dev = torch.zeros(blk.cap_nodes[-1], dims[0], dtype=torch.float32, device="cuda")
    x_dev[:len(x)] = torch.from_numpy(x).cuda()
    logits = torch.full((blk.cap_nodes[0], dims[-1]), float("nan"), dtype=torch.float32, device="cuda")
    dci.dci_sage_forward(ctx, blk, x_dev, [gu.dev(a) for a in ws], [gu.dev(a) for a in wn], [gu.dev(a) for a in bs],
                         logits)
    ctx.sync()
    _logit_check(logits[:n_seeds].cpu().numpy(), want)


@pytest.mark.parametrize("model", [0, 1, 2])
@pytest.mark.parametrize("dims,fanouts,n_seeds", [((64, 64, 16), (5, 10), 256), ((100, 130, 47), (3, 4), 70),
                                                  ((63, 5), (7,), 129), ((602, 256, 256, 41), (2, 3, 4), 33)])
def test_gnn_forward_model_variants_match_oracle(env, model, dims, fanouts, n_seeds):
    """GraphSAGE-mean, GraphSAGE-sum and GCN-avg (Table III); input widths of 63, 100 and 130 give the
    one-operand product of the GCN layer an odd number of 16-wide slabs."""
    dci, gu, ctx, g, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "graph", "tiny", "w"))
    seeds = tiny["seeds"][:n_seeds]
    want_blk = oracle.sample_khop(tiny["indptr"], tiny["indices"], seeds, 2, fanouts, 6)
    blk = dci.Blocks(ctx, w.num_nodes, n_seeds, fanouts)
    dci.dci_sample_khop(ctx, g, None, gu.dev(seeds), 2, fanouts, 6, blk)
    feat = synth.features(w.num_nodes, dims[0], 41)
    ws, wn, bs = synth.sage_weights(dims, 42)
    x = feat[want_blk.nodes]
    want = oracle.gnn_forward(model, want_blk, x, ws, wn, bs)
    x_dev = torch.zeros(blk.cap_nodes[-1], dims[0], dtype=torch.float32, device="cuda")
    x_dev[:len(x)] = torch.from_numpy(x).cuda()
    logits = torch.full((blk.cap_nodes[0], dims[-1]), float("nan"), dtype=torch.float32, device="cuda")
    dci.dci_gnn_forward(ctx, blk, x_dev, model, None if model == 2 else [gu.dev(a) for a in ws],
                        [gu.dev(a) for a in wn], [gu.dev(a) for a in bs], logits)
    ctx.sync()
    _logit_check(logits[:n_seeds].cpu().numpy(), want)


@pytest.mark.parametrize("model", [0, 1, 2])
def test_gnn_forward_with_empty_rows(env, small_graphs, model):
    dci, gu, ctx = env["dci"], env["gu"], env["ctx"]
    indptr, indices = small_graphs[3]          # isolated nodes, a self loop, a duplicated edge
    g = gu.make_graph(indptr, indices, None)
    seeds = np.array([0, 4, 1, 3, 2], dtype=np.int64)
    dims, fanouts = (6, 9, 3), (3, 2)
    want_blk = oracle.sample_khop(indptr, indices, seeds, 0, fanouts, 4)
    assert (np.diff(want_blk.blk_indptr[0]) == 0).any()
    blk = dci.Blocks(ctx, 5, len(seeds), fanouts)
    dci.dci_sample_khop(ctx, g, None, gu.dev(seeds), 0, fanouts, 4, blk)
    x = synth.features(5, dims[0], 51)[want_blk.nodes]
    ws, wn, bs = synth.sage_weights(dims, 52)
    want = oracle.gnn_forward(model, want_blk, x, ws, wn, bs)
    x_dev = torch.zeros(blk.cap_nodes[-1], dims[0], dtype=torch.float32, device="cuda")
    x_dev[:len(x)] = torch.from_numpy(x).cuda()
    logits = torch.full((blk.cap_nodes[0], dims[-1]), float("nan"), dtype=torch.float32, device="cuda")
    dci.dci_gnn_forward(ctx, blk, x_dev, model, [gu.dev(a) for a in ws], [gu.dev(a) for a in wn],
                        [gu.dev(a) for a in bs], logits)
    ctx.sync()
    _logit_check(logits[:len(seeds)].cpu().numpy(), want)


def _forward_case(env, dims, fanouts, n_seeds, model, option, batch=3, rng_seed=8):
    dci, gu, ctx, g, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "graph", "tiny", "w"))
    seeds = tiny["seeds"][:n_seeds]
    want_blk = oracle.sample_khop(tiny["indptr"], tiny["indices"], seeds, batch, fanouts, rng_seed)
    blk = dci.Blocks(ctx, w.num_nodes, n_seeds, fanouts)
    dci.dci_sample_khop(ctx, g, None, gu.dev(seeds), batch, fanouts, rng_seed, blk)
    feat = synth.features(w.num_nodes, dims[0], 61)
    ws, wn, bs = synth.sage_weights(dims, 62)
    x = feat[want_blk.nodes]
    want = oracle.gnn_forward(model, want_blk, x, ws, wn, bs)
    x_dev = torch.zeros(blk.cap_nodes[-1], dims[0], dtype=torch.float32, device="cuda")
    x_dev[:len(x)] = torch.from_numpy(x).cuda()
    logits = torch.full((blk.cap_nodes[0], dims[-1]), float("nan"), dtype=torch.float32, device="cuda")
    ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, option)
    try:
        dci.dci_gnn_forward(ctx, blk, x_dev, model, [gu.dev(a) for a in ws], [gu.dev(a) for a in wn],
                            [gu.dev(a) for a in bs], logits)
        ctx.sync()
    finally:
        ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, 0)
    _logit_check(logits[:n_seeds].cpu().numpy(), want)
    return [int(v) for v in want_blk.n_nodes]


@pytest.mark.parametrize("model", [0, 2])
@pytest.mark.parametrize("dims,fanouts,n_seeds", [((602, 256, 128), (3, 4), 70), ((100, 128, 256, 47), (2, 3, 4), 33),
                                                  ((8, 128), (7,), 129), ((16, 128), (5,), 1), ((48, 128, 128), (5, 5), 300),
                                                  ((256, 512, 384), (10, 25), 40)])
def test_wide_linear_kernel_matches_oracle(env, model, dims, fanouts, n_seeds):
    """The wide dense-layer kernel forced on at small sizes: input widths with and without a k tail (602, 100, 8),
    fewer k-slabs than pipeline stages (8, 16, 48), one to four column tiles, both operand counts."""
    _forward_case(env, dims, fanouts, n_seeds, model, option=2)


@pytest.mark.parametrize("model", [0, 2])
@pytest.mark.parametrize("dims,fanouts,n_seeds", [((602, 256, 128), (3, 4), 70), ((100, 64, 192, 64), (2, 3, 4), 33),
                                                  ((8, 64), (7,), 129), ((16, 128), (5,), 1), ((48, 64, 64), (5, 5), 300),
                                                  ((256, 512, 320), (10, 25), 40)])
def test_dma_tile_kernel_matches_oracle(env, model, dims, fanouts, n_seeds):
    """The 64x64 kernel fed by global->LDS loads (kernel choice 3, contraction not split): input widths with and
    without a k tail, fewer k-slabs than pipeline stages, one to eight column tiles, both operand counts."""
    dci, ctx = env["dci"], env["ctx"]
    ctx.set_option(dci.DCI_OPT_LINEAR_SPLIT, 1)
    try:
        _forward_case(env, dims, fanouts, n_seeds, model, option=3)
    finally:
        ctx.set_option(dci.DCI_OPT_LINEAR_SPLIT, 0)


@pytest.mark.parametrize("option", [0, 1, 3])
def test_forward_many_rows(env, option):
    """A layer tall enough for the default choice to take the wide kernel with several row blocks per workgroup
    (option 0), against the same through the tile kernel (option 1)."""
    n_nodes = _forward_case(env, (192, 256, 128, 16), (8, 8, 8), 2048, 0, option)
    assert n_nodes[2] > 4096      # more than one 32-row block for each of the 128 workgroups of a column tile


@pytest.mark.parametrize("M,K,N", [(60000, 40, 128), (120000, 40, 256)])
def test_wide_linear_kernel_in_several_passes(env, M, K, N):
    """More than six 32-row blocks per workgroup: 60,000 rows through one 128-column tile over 256 workgroups (two
    passes of four blocks) and 120,000 rows through two tiles over 128 workgroups each (five passes of six).
    The block has no edges, so the layer is x W_self + b; the neighbour operand (all zeros) still takes the same path."""
    dci, gu, ctx = env["dci"], env["gu"], env["ctx"]
    blk = dci.Blocks(ctx, 10**6, M, (1,))
    assert blk.cap_nodes[0] >= M
    blk.counts.zero_()
    blk.counts[0] = M
    blk.counts[1] = M
    blk.blk_indptr[0].zero_()
    rng = np.random.default_rng(9)
    x = rng.standard_normal((M, K), dtype=np.float32)
    ws, wn, bs = synth.sage_weights((K, N), 63)
    want_blk = oracle.Blocks(n_nodes=np.array([M, M]), n_edges=np.array([0]), nodes=np.arange(M, dtype=np.int64),
                             blk_indptr=[np.zeros(M + 1, dtype=np.int64)], blk_src=[np.zeros(0, dtype=np.int32)],
                             src_global=[np.zeros(0, dtype=np.int64)], src_pos=[np.zeros(0, dtype=np.int64)])
    want = oracle.gnn_forward(0, want_blk, x, ws, wn, bs)
    x_dev = torch.zeros(blk.cap_nodes[1], K, dtype=torch.float32, device="cuda")
    x_dev[:M] = torch.from_numpy(x).cuda()
    logits = torch.full((blk.cap_nodes[0], N), float("nan"), dtype=torch.float32, device="cuda")
    ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, 2)     # the input is narrower than the default choice asks for
    try:
        dci.dci_sage_forward(ctx, blk, x_dev, [gu.dev(a) for a in ws], [gu.dev(a) for a in wn], [gu.dev(a) for a in bs], logits)
        ctx.sync()
    finally:
        ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, 0)
    _logit_check(logits[:M].cpu().numpy(), want)


def test_dense_layer_kernels_on_random_shapes(env):
    """Forty random layer shapes through every kernel choice: row counts around the 32- and 64-row tile edges,
    input widths from 1 to 330 (k tails, fewer slabs than pipeline stages, odd widths), output widths that are and
    are not multiples of 64 / 128.  One block without edges for the two-operand layer (x W_self + b) and the GCN
    layer (x W + b, the row itself being its only aggregate)."""
    dci, gu, ctx = env["dci"], env["gu"], env["ctx"]
    rng = np.random.default_rng(77)
    widths_out = [1, 5, 41, 47, 64, 100, 128, 172, 192, 256, 320, 384]
    for case in range(40):
        M = int(rng.choice([1, 31, 32, 33, 63, 64, 65, 200, 1000, 2049, 3000]))
        K = int(rng.choice([1, 2, 7, 8, 15, 16, 17, 31, 32, 48, 63, 64, 100, 130, 256, 330]))
        N = int(rng.choice(widths_out))
        model = int(rng.choice([0, 2]))
        option = int(rng.choice([0, 1, 2, 3]))
        split = int(rng.choice([0, 1]))
        if case % 4 == 3:
            option = 4   # weights in registers, where the shape allows it (else the default choice)
        blk = dci.Blocks(ctx, 10**6, M, (1,))
        blk.counts.zero_()
        blk.counts[0] = M
        blk.counts[1] = M
        blk.blk_indptr[0].zero_()
        x = rng.standard_normal((M, K), dtype=np.float32)
        ws, wn, bs = synth.sage_weights((K, N), 100 + case)
        want_blk = oracle.Blocks(n_nodes=np.array([M, M]), n_edges=np.array([0]), nodes=np.arange(M, dtype=np.int64),
                                 blk_indptr=[np.zeros(M + 1, dtype=np.int64)], blk_src=[np.zeros(0, dtype=np.int32)],
                                 src_global=[np.zeros(0, dtype=np.int64)], src_pos=[np.zeros(0, dtype=np.int64)])
        want = oracle.gnn_forward(model, want_blk, x, ws, wn, bs)
        x_dev = torch.zeros(blk.cap_nodes[1], K, dtype=torch.float32, device="cuda")
        x_dev[:M] = torch.from_numpy(x).cuda()
        logits = torch.full((blk.cap_nodes[0], N), float("nan"), dtype=torch.float32, device="cuda")
        ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, option)
        ctx.set_option(dci.DCI_OPT_LINEAR_SPLIT, split)
        try:
            dci.dci_gnn_forward(ctx, blk, x_dev, model, [gu.dev(a) for a in ws], [gu.dev(a) for a in wn],
                                [gu.dev(a) for a in bs], logits)
            ctx.sync()
        finally:
            ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, 0)
            ctx.set_option(dci.DCI_OPT_LINEAR_SPLIT, 0)
        got = logits.cpu().numpy()
        tol = 1e-4 * max(1.0, float(np.abs(want).max()))
        err = float(np.abs(got[:M].astype(np.float64) - want).max())
        assert err <= tol, f"case {case}: M={M} K={K} N={N} model={model} kernel={option} split={split}: {err} > {tol}"
        assert np.isnan(got[M:]).all(), f"case {case}: rows beyond the batch were written"


@pytest.mark.parametrize("model", [0, 2])
@pytest.mark.parametrize("dims,fanouts,n_seeds", [((128, 256, 256), (3, 4), 70), ((100, 256, 47), (5, 5), 256),
                                                  ((4, 256), (7,), 129), ((8, 512), (5,), 1), ((124, 256, 256), (5, 5), 300),
                                                  ((64, 512, 256), (10, 25), 40)])
def test_resident_weights_kernel_matches_oracle(env, model, dims, fanouts, n_seeds):
    """The dense-layer kernel that keeps the weights in registers (kernel choice 4) forced on at small sizes:
    contractions that fill all sixteen slabs (2 x 128), end inside a slab (2 x 100, 2 x 124, 2 x 4) or, for the
    one-operand GCN layer, are half as long; one and two 256-column tiles; a single row and row counts that leave
    the last 32-row block ragged; layers it cannot take (47 outputs, 512 inputs) fall back to the other kernels."""
    _forward_case(env, dims, fanouts, n_seeds, model, option=4)


def test_resident_weights_kernel_many_blocks(env):
    """More 32-row blocks than workgroups (every workgroup walks several blocks, the three row buffers wrap, both
    accumulator sets are stored) with a ragged last block, for both operand counts and a contraction that ends
    inside a slab."""
    dci, gu, ctx = env["dci"], env["gu"], env["ctx"]
    rng = np.random.default_rng(5)
    for M, K, N, model in ((40_001, 100, 256, 0), (33_000, 128, 256, 0), (24_577, 200, 512, 2)):
        blk = dci.Blocks(ctx, 10**6, M, (1,))
        blk.counts.zero_()
        blk.counts[0] = M
        blk.counts[1] = M
        blk.blk_indptr[0].zero_()
        x = rng.standard_normal((M, K), dtype=np.float32)
        ws, wn, bs = synth.sage_weights((K, N), 300 + K)
        want_blk = oracle.Blocks(n_nodes=np.array([M, M]), n_edges=np.array([0]), nodes=np.arange(M, dtype=np.int64),
                                 blk_indptr=[np.zeros(M + 1, dtype=np.int64)], blk_src=[np.zeros(0, dtype=np.int32)],
                                 src_global=[np.zeros(0, dtype=np.int64)], src_pos=[np.zeros(0, dtype=np.int64)])
        want = oracle.gnn_forward(model, want_blk, x, ws, wn, bs)
        x_dev = torch.zeros(blk.cap_nodes[1], K, dtype=torch.float32, device="cuda")
        x_dev[:M] = torch.from_numpy(x).cuda()
        logits = torch.full((blk.cap_nodes[0], N), float("nan"), dtype=torch.float32, device="cuda")
        ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, 4)
        try:
            dci.dci_gnn_forward(ctx, blk, x_dev, model, [gu.dev(a) for a in ws], [gu.dev(a) for a in wn],
                                [gu.dev(a) for a in bs], logits)
            ctx.sync()
        finally:
            ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, 0)
        got = logits.cpu().numpy()
        tol = 1e-4 * max(1.0, float(np.abs(want).max()))
        err = float(np.abs(got[:M].astype(np.float64) - want).max())
        assert err <= tol, f"M={M} K={K} N={N} model={model}: {err} > {tol}"
        assert np.isnan(got[M:]).all()


@pytest.mark.parametrize("split", [1, 2, 0])
def test_split_contraction_matches_oracle(env, split):
    """Few tiles: by default (0) the 64x64 kernel shares each tile between up to eight workgroups and a second
    kernel adds their partial sums; 1 switches that off, 2 limits it to two."""
    dci, ctx = env["dci"], env["ctx"]
    ctx.set_option(dci.DCI_OPT_LINEAR_SPLIT, split)
    try:
        for model in (0, 2):
            _forward_case(env, (602, 256, 41), (3, 4), 70, model, option=1)
            _forward_case(env, (100, 130, 47), (5, 5), 256, model, option=1)
    finally:
        ctx.set_option(dci.DCI_OPT_LINEAR_SPLIT, 0)


def test_set_option_rejects_bad_values(env):
    dci, ctx = env["dci"], env["ctx"]
    with pytest.raises(dci.DciError):
        ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, 5)
    with pytest.raises(dci.DciError):
        ctx.set_option(dci.DCI_OPT_LINEAR_SPLIT, 9)
    with pytest.raises(dci.DciError):
        ctx.set_option(dci.DCI_OPT_INPUT_LAYER, 4)
    with pytest.raises(dci.DciError):
        ctx.set_option(99, 0)


def test_gnn_forward_rejects_bad_arguments(env):
    dci, gu, ctx, g, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "graph", "tiny", "w"))
    blk = dci.Blocks(ctx, w.num_nodes, 8, (2,))
    dci.dci_sample_khop(ctx, g, None, gu.dev(tiny["seeds"][:8]), 0, (2,), 1, blk)
    ws, wn, bs = ([gu.dev(a) for a in t] for t in synth.sage_weights((16, 4), 1))
    x = torch.zeros(blk.cap_nodes[-1], 16, dtype=torch.float32, device="cuda")
    logits = torch.zeros(8, 4, dtype=torch.float32, device="cuda")
    with pytest.raises(dci.DciError):
        dci.dci_gnn_forward(ctx, blk, x, 3, ws, wn, bs, logits)
    with pytest.raises(dci.DciError):
        dci.dci_gnn_forward(ctx, blk, x, 0, None, wn, bs, logits)   # GraphSAGE needs both weight sets


def test_end_to_end_tiny(env):
    """presample -> fill -> sample -> gather -> forward, all on the GPU, against the oracle."""
    dci, gu, ctx, g, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "graph", "tiny", "w"))
    seeds = gu.dev(tiny["seeds"])
    fc = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
    ac = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
    dci.dci_presample_count(ctx, g, None, seeds, w.batch_size, 0, w.n_presample, w.presample_first_batch, w.fanouts,
                            w.rng_seed, fc, ac)
    cache = dci.dci_fill_caches(ctx, g, fc, ac, w.budget_bytes, 3, 7, 0)
    oc = _oracle_caches(tiny, w)
    assert np.array_equal(cache.adj_remap.cpu().numpy(), oc["adj_remap"])
    assert np.array_equal(cache.feat_remap.cpu().numpy(), oc["feat_remap"])
    blk = dci.Blocks(ctx, w.num_nodes, w.batch_size, w.fanouts)
    x = torch.empty(blk.cap_nodes[-1], w.feat_dim, dtype=torch.float32, device="cuda")
    logits = torch.empty(w.batch_size, w.classes, dtype=torch.float32, device="cuda")
    ws, wn, bs = ([gu.dev(a) for a in tiny[k]] for k in ("w_self", "w_neigh", "bias"))
    for b in range(w.num_batches):
        sl = slice(b * w.batch_size, (b + 1) * w.batch_size)
        stats = gu.new_stats()
        dci.dci_sample_khop(ctx, g, cache, seeds[sl], b, w.fanouts, w.rng_seed, blk, stats)
        dci.dci_gather_features(ctx, g, cache, blk.nodes, blk.cap_nodes[-1], x, n_dev=blk.n_input_dev(), stats=stats)
        dci.dci_sage_forward(ctx, blk, x, ws, wn, bs, logits)
        got = gu.blocks_to_host(ctx, blk)
        want_blk = oracle.sample_khop(tiny["indptr"], tiny["indices"], tiny["seeds"][sl], b, w.fanouts, w.rng_seed)
        gu.assert_blocks_equal(got, want_blk)
        n_in = got["n_nodes"][-1]
        want_x = oracle.gather(tiny["feat"], want_blk.nodes)
        assert x[:n_in].cpu().numpy().tobytes() == want_x.tobytes()
        want = oracle.sage_forward(want_blk, want_x, tiny["w_self"], tiny["w_neigh"], tiny["bias"])
        _logit_check(logits.cpu().numpy(), want)
        st = gu.stats_dict(ctx, stats)
        assert st["feat_hits"] == int((oc["feat_remap"][want_blk.nodes] >= 0).sum())
        assert st["feat_hits"] + st["feat_misses"] == n_in


def _host_lines(base_ptr, byte_offsets):
    """Distinct 128-byte lines among the addresses base_ptr + byte_offsets."""
    return len(np.unique((base_ptr + np.asarray(byte_offsets, dtype=np.int64)) >> 7))


def _expected_sampler_traffic(want, fanouts, indptr, adj_remap, indptr_base, indices_base):
    """(bytes_hbm, bytes_host, lines_bounds, lines_ids) of sampling the batch `want` through a node-granular adjacency
    cache, from the oracle's blocks and sampled positions: 16 bytes of list bounds per frontier node and
    8 bytes per neighbour id, charged to the tier that serves the node; lines = per missed node, the lines
    of its two list bounds (only at the hop at which the node joins the frontier: the sampler notes them for the
    batch's later hops) plus the distinct lines of the neighbour ids it reads."""
    b_hbm = b_host = lines = blines = 0
    for h in range(len(fanouts)):
        frontier = want.nodes[:want.n_nodes[h]]
        hit = adj_remap[frontier] >= 0 if adj_remap is not None else np.zeros(len(frontier), dtype=bool)
        bi = want.blk_indptr[h]
        rows = np.diff(bi)
        b_hbm += 16 * int(hit.sum()) + 8 * int(rows[hit].sum())
        b_host += 16 * int((~hit).sum()) + 8 * int(rows[~hit].sum())
        n_noted = int(want.n_nodes[h - 1]) if h > 0 else 0   # these rows' bounds were fetched at an earlier hop
        for i in np.flatnonzero(~hit):
            v = int(frontier[i])
            if i >= n_noted:
                blines += _host_lines(indptr_base, [8 * v, 8 * (v + 1)])
            pos = want.src_pos[h][bi[i]:bi[i + 1]]
            if len(pos):
                lines += _host_lines(indices_base, 8 * (int(indptr[v]) + pos))
    return b_hbm, b_host, blines, lines


@pytest.mark.parametrize("with_cache", [False, True])
def test_traffic_statistics_match_counts_derived_from_the_oracle(env, with_cache):
    """bytes_hbm / bytes_host / host_lines of sampling and gathering, exact."""
    dci, gu, ctx, g, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "graph", "tiny", "w"))
    oc = _oracle_caches(tiny, w) if with_cache else None
    cache = gu.upload_cache(oc["adj_remap"], oc["c_indptr"], oc["c_indices"], oc["feat_remap"], oc["feat_cache"]) if oc else None
    blk = dci.Blocks(ctx, w.num_nodes, w.batch_size, w.fanouts)
    x = torch.empty(blk.cap_nodes[-1], w.feat_dim, dtype=torch.float32, device="cuda")
    for b, fan in ((1, w.fanouts), (6, (12, 3))):
        seeds = tiny["seeds"][b * w.batch_size:(b + 1) * w.batch_size]
        blk = dci.Blocks(ctx, w.num_nodes, w.batch_size, fan)
        stats = gu.new_stats()
        dci.dci_sample_khop(ctx, g, cache, gu.dev(seeds), b, fan, w.rng_seed, blk, stats)
        st = gu.stats_dict(ctx, stats)
        want = oracle.sample_khop(tiny["indptr"], tiny["indices"], seeds, b, fan, w.rng_seed)
        gu.assert_blocks_equal(gu.blocks_to_host(ctx, blk), want)
        exp = _expected_sampler_traffic(want, fan, tiny["indptr"], oc["adj_remap"] if oc else None,
                                        g.indptr.data_ptr(), g.indices.data_ptr())
        assert (st["bytes_hbm"], st["bytes_host"], st["lines_bounds"], st["lines_ids"]) == exp
        assert exp[2] > 0 and exp[3] > 0 and (exp[0] > 0) == with_cache
        # the gather adds one row of 4F bytes per input node to the tier that holds it
        n_in = int(want.n_nodes[-1])
        dci.dci_gather_features(ctx, g, cache, blk.nodes, n_in, x, stats=stats)
        st2 = gu.stats_dict(ctx, stats)
        hits = int((oc["feat_remap"][want.nodes] >= 0).sum()) if oc else 0
        assert st2["bytes_hbm"] - st["bytes_hbm"] == 4 * w.feat_dim * hits
        assert st2["bytes_host"] - st["bytes_host"] == 4 * w.feat_dim * (n_in - hits)
        assert (st2["lines_bounds"], st2["lines_ids"]) == (st["lines_bounds"], st["lines_ids"])


def test_relabel_timeout_voids_the_batch_and_is_reported(env):
    """The frontier scan's give-up path, forced from the host: tiles are numbered from 1, so tile 0 never
    exists and never publishes; with the spin limit at 200 polls every kernel still ends at once.  The next
    dci_sync reports the failure, the batch's sizes are zero, a following gather / forward touches nothing,
    and the context works again once the hook is off."""
    dci, gu, g, tiny, w = (env[k] for k in ("dci", "gu", "graph", "tiny", "w"))
    ctx = dci.Context(0, workspace_bytes=64 << 20)     # large enough for all three calls: growing it would sync
    n = 600                                            # three scan tiles at hop 0 (256 rows each)
    seeds = tiny["seeds"][:n]
    blk = dci.Blocks(ctx, w.num_nodes, n, w.fanouts)
    with pytest.raises(dci.DciError) as e:             # the hook is refused while the limit is at its default
        ctx.set_option(dci.DCI_OPT_TEST_RELABEL_FIRST_TICKET, 1)
    assert e.value.code == -1
    ctx.set_option(dci.DCI_OPT_RELABEL_SPIN_LIMIT, 200)
    ctx.set_option(dci.DCI_OPT_TEST_RELABEL_FIRST_TICKET, 1)
    with pytest.raises(dci.DciError) as e:
        ctx.set_option(dci.DCI_OPT_RELABEL_SPIN_LIMIT, 1 << 24)
    assert e.value.code == -1
    ws, wn, bs = ([gu.dev(a) for a in tiny[k]] for k in ("w_self", "w_neigh", "bias"))
    x = torch.full((blk.cap_nodes[-1], w.feat_dim), 7.0, dtype=torch.float32, device="cuda")
    logits = torch.full((n, w.classes), 9.0, dtype=torch.float32, device="cuda")
    stats = gu.new_stats()
    for first in (1, 40):                              # 40: every numbered tile lies beyond the frontier
        ctx.set_option(dci.DCI_OPT_TEST_RELABEL_FIRST_TICKET, first)
        blk.counts.fill_(123)
        dci.dci_sample_khop(ctx, g, None, gu.dev(seeds), 0, w.fanouts, w.rng_seed, blk, stats)
        dci.dci_gather_features(ctx, g, None, blk.nodes, blk.cap_nodes[-1], x, n_dev=blk.n_input_dev())
        dci.dci_sage_forward(ctx, blk, x, ws, wn, bs, logits)
        with pytest.raises(dci.DciError) as e:
            ctx.sync()
        assert e.value.code == -3 and "relabel scan timed out" in str(e.value)
        ctx.sync()                                     # reported once
        assert blk.counts.cpu().numpy().tolist() == [0] * 17 and blk.counts_host.numpy().tolist() == [0] * 17
        assert bool((x == 7.0).all()) and bool((logits == 9.0).all())
        assert stats.cpu().numpy().tolist() == [0] * dci.STATS_WORDS
    ctx.set_option(dci.DCI_OPT_TEST_RELABEL_FIRST_TICKET, 0)
    ctx.set_option(dci.DCI_OPT_RELABEL_SPIN_LIMIT, 1 << 24)
    dci.dci_sample_khop(ctx, g, None, gu.dev(seeds), 0, w.fanouts, w.rng_seed, blk, stats)
    gu.assert_blocks_equal(gu.blocks_to_host(ctx, blk), oracle.sample_khop(tiny["indptr"], tiny["indices"], seeds, 0,
                                                                            w.fanouts, w.rng_seed))


@pytest.mark.parametrize("F,model", [(64, 0), (64, 2), (63, 0), (602, 0), (602, 1), (100, 2), (1, 0), (130, 0)])
def test_gather_forward_reads_cached_rows_in_place(env, F, model):
    """dci_gather_forward against the oracle and against dci_gather_features + dci_gnn_forward: the same logits
    bit for bit (the sums run in the same order), the same hit / miss statistics, and in x only the rows that
    miss or belong to F_{L-1}; with a partly filled feature cache, with none, and with everything cached."""
    dci, gu, ctx, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "tiny", "w"))
    N = w.num_nodes
    feat = synth.features(N, F, 40 + F)
    g = gu.make_graph(tiny["indptr"], tiny["indices"], feat)
    dims = (F, 48, 10)
    ws_h, wn_h, b_h = synth.sage_weights(dims, 77)
    ws, wn, bs = ([gu.dev(a) for a in arr] for arr in (ws_h, wn_h, b_h))
    rng = np.random.default_rng(F * 10 + model)
    seeds = tiny["seeds"][300:300 + 200]
    want = oracle.sample_khop(tiny["indptr"], tiny["indices"], seeds, 5, w.fanouts, w.rng_seed)
    want_x = oracle.gather(feat, want.nodes)
    ref = oracle.gnn_forward(model, want, want_x, ws_h, wn_h, b_h)
    n_in, n_dense = len(want.nodes), int(want.n_nodes[w.n_hops - 1])
    for share in (0.5, None, 1.0):
        if share is None:
            cache, remap = None, np.full(N, -1, dtype=np.int32)
        else:
            k = int(N * share)
            rows = rng.permutation(N)[:k]
            remap = np.full(N, -1, dtype=np.int32)
            remap[rows] = np.arange(k, dtype=np.int32)
            cache = gu.upload_cache(np.full(N, -1), np.zeros(1, np.int64), np.zeros(0, np.int64), remap, feat[rows])
        blk = dci.Blocks(ctx, N, len(seeds), w.fanouts)
        dci.dci_sample_khop(ctx, g, cache, gu.dev(seeds), 5, w.fanouts, w.rng_seed, blk)
        x = torch.full((blk.cap_nodes[-1], F), -123.0, dtype=torch.float32, device="cuda")
        logits = torch.zeros(len(seeds), dims[-1], dtype=torch.float32, device="cuda")
        stats = gu.new_stats()
        dci.dci_gather_forward(ctx, g, cache, blk, x, model, None if model == 2 else ws, wn, bs, logits, stats)
        st = gu.stats_dict(ctx, stats)
        got = logits.cpu().numpy()
        _logit_check(got, ref)
        hit = remap[want.nodes] >= 0
        assert (st["feat_hits"], st["feat_misses"]) == (int(hit.sum()), int((~hit).sum()))
        assert (st["bytes_hbm"], st["bytes_host"]) == (4 * F * int(hit.sum()), 4 * F * int((~hit).sum()))
        xs = x.cpu().numpy()
        copied = ~hit | (np.arange(n_in) < n_dense)
        assert st["rows_copied"] == int(copied.sum())
        assert xs[:n_in][copied].tobytes() == want_x[copied].tobytes()
        assert (xs[:n_in][~copied] == -123.0).all() and (xs[n_in:] == -123.0).all()
        if share == 0.5:
            assert 0 < copied.sum() < n_in
        # the two-call route gives the same bits
        x2 = torch.empty_like(x)
        logits2 = torch.zeros_like(logits)
        dci.dci_gather_features(ctx, g, cache, blk.nodes, blk.cap_nodes[-1], x2, n_dev=blk.n_input_dev())
        dci.dci_gnn_forward(ctx, blk, x2, model, None if model == 2 else ws, wn, bs, logits2)
        ctx.sync()
        assert logits2.cpu().numpy().tobytes() == got.tobytes()


@pytest.mark.parametrize("F,hidden,fanouts,model,n_seeds", [(128, 256, (5, 10), 0, 200), (100, 256, (5, 10), 1, 333),
                                                            (64, 512, (3, 16), 0, 97), (4, 256, (2, 25), 0, 150),
                                                            (124, 256, (4, 40), 1, 64), (128, 256, (7,), 0, 1)])
def test_input_layer_in_one_kernel_matches_the_two_kernel_route(env, F, hidden, fanouts, model, n_seeds):
    """The first layer as one kernel (aggregation inside the weights-in-registers dense layer, forced on at small sizes)
    against the oracle, and bit for bit against the aggregation kernel followed by the same dense kernel: widths that fill
    all sixteen slabs and that end inside one, one and two 256-column tiles, rows with more edges than the sixteen the
    pipelined part takes (fan-outs 25 and 40), empty rows, a single seed, with a partly filled feature cache (rows read in
    place through dci_gather_forward) and with none (dci_gnn_forward on gathered rows)."""
    dci, gu, ctx, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "tiny", "w"))
    N = w.num_nodes
    feat = synth.features(N, F, 90 + F)
    g = gu.make_graph(tiny["indptr"], tiny["indices"], feat)
    dims = (F, hidden) if len(fanouts) == 1 else (F, hidden, 10)
    ws_h, wn_h, b_h = synth.sage_weights(dims, 78)
    ws, wn, bs = ([gu.dev(a) for a in arr] for arr in (ws_h, wn_h, b_h))
    seeds = tiny["seeds"][100:100 + n_seeds]
    want = oracle.sample_khop(tiny["indptr"], tiny["indices"], seeds, 9, fanouts, w.rng_seed)
    want_x = oracle.gather(feat, want.nodes)
    ref = oracle.gnn_forward(model, want, want_x, ws_h, wn_h, b_h)
    rng = np.random.default_rng(F)
    rows = rng.permutation(N)[:N // 2]
    remap = np.full(N, -1, dtype=np.int32)
    remap[rows] = np.arange(len(rows), dtype=np.int32)
    cache = gu.upload_cache(np.full(N, -1), np.zeros(1, np.int64), np.zeros(0, np.int64), remap, feat[rows])
    blk = dci.Blocks(ctx, N, len(seeds), fanouts)
    dci.dci_sample_khop(ctx, g, cache, gu.dev(seeds), 9, fanouts, w.rng_seed, blk)
    out = {}
    for kind in (2, 1):
        ctx.set_option(dci.DCI_OPT_INPUT_LAYER, kind)
        ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, 4)   # the two-kernel route then ends in the same dense kernel
        try:
            x = torch.full((blk.cap_nodes[-1], F), -7.0, dtype=torch.float32, device="cuda")
            l1 = torch.zeros(len(seeds), dims[-1], dtype=torch.float32, device="cuda")
            dci.dci_gather_forward(ctx, g, cache, blk, x, model, ws, wn, bs, l1)
            x2 = torch.empty_like(x)
            l2 = torch.zeros_like(l1)
            dci.dci_gather_features(ctx, g, cache, blk.nodes, blk.cap_nodes[-1], x2, n_dev=blk.n_input_dev())
            dci.dci_gnn_forward(ctx, blk, x2, model, ws, wn, bs, l2)
            ctx.sync()
        finally:
            ctx.set_option(dci.DCI_OPT_INPUT_LAYER, 0)
            ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, 0)
        out[kind] = (l1.cpu().numpy(), l2.cpu().numpy())
        _logit_check(out[kind][0], ref)
        _logit_check(out[kind][1], ref)
    assert out[2][0].tobytes() == out[1][0].tobytes()
    assert out[2][1].tobytes() == out[1][1].tobytes()
    assert out[2][0].tobytes() == out[2][1].tobytes()


@pytest.mark.parametrize("F,hidden,fanouts,model,n_seeds,room", [(128, 256, (5, 10), 0, 200, 1), (112, 320, (5, 10), 1, 333, 1),
                                                                 (64, 512, (3, 16), 0, 97, 1), (32, 64, (2, 25), 0, 150, 1),
                                                                 (48, 192, (4, 40), 1, 64, 1), (128, 256, (7,), 0, 1, 1),
                                                                 (128, 256, (5, 10), 0, 200, 3), (64, 384, (3, 16), 0, 97, 4)])
def test_input_layer_in_one_kernel_of_64_row_tiles(env, F, hidden, fanouts, model, n_seeds, room):
    """The first layer as one kernel in its other form (half of a workgroup aggregates 64 rows into LDS while the other
    half multiplies the 64 before), forced on at small sizes: against the oracle, and - where the output width allows
    that kernel - bit for bit against the aggregation kernel followed by the weights-in-registers dense kernel, whose
    order of summation it shares.  Two to eight slabs per operand, output widths that end inside a pass of 128 columns,
    rows with more edges than the sixteen loaded at once, empty rows, a last tile of one row, cached rows read in place
    and gathered rows; with `room` > 1 the batch's buffers are sized for `room` times as many seeds, so that the launch has
    more than twice as many workgroups as tiles and two workgroups share every tile (one half of the passes each)."""
    dci, gu, ctx, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "tiny", "w"))
    N = w.num_nodes
    feat = synth.features(N, F, 190 + F)
    g = gu.make_graph(tiny["indptr"], tiny["indices"], feat)
    dims = (F, hidden) if len(fanouts) == 1 else (F, hidden, 10)
    ws_h, wn_h, b_h = synth.sage_weights(dims, 79)
    ws, wn, bs = ([gu.dev(a) for a in arr] for arr in (ws_h, wn_h, b_h))
    seeds = tiny["seeds"][50:50 + n_seeds]
    want = oracle.sample_khop(tiny["indptr"], tiny["indices"], seeds, 11, fanouts, w.rng_seed)
    want_x = oracle.gather(feat, want.nodes)
    ref = oracle.gnn_forward(model, want, want_x, ws_h, wn_h, b_h)
    rng = np.random.default_rng(F + 1)
    rows = rng.permutation(N)[:N // 2]
    remap = np.full(N, -1, dtype=np.int32)
    remap[rows] = np.arange(len(rows), dtype=np.int32)
    cache = gu.upload_cache(np.full(N, -1), np.zeros(1, np.int64), np.zeros(0, np.int64), remap, feat[rows])
    blk = dci.Blocks(ctx, N, room * len(seeds), fanouts)
    dci.dci_sample_khop(ctx, g, cache, gu.dev(seeds), 11, fanouts, w.rng_seed, blk)
    out = {}
    for kind in (3, 1):
        ctx.set_option(dci.DCI_OPT_INPUT_LAYER, kind)
        ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, 4)
        try:
            x = torch.full((blk.cap_nodes[-1], F), -7.0, dtype=torch.float32, device="cuda")
            l1 = torch.zeros(room * len(seeds), dims[-1], dtype=torch.float32, device="cuda")
            dci.dci_gather_forward(ctx, g, cache, blk, x, model, ws, wn, bs, l1)
            x2 = torch.empty_like(x)
            l2 = torch.zeros_like(l1)
            dci.dci_gather_features(ctx, g, cache, blk.nodes, blk.cap_nodes[-1], x2, n_dev=blk.n_input_dev())
            dci.dci_gnn_forward(ctx, blk, x2, model, ws, wn, bs, l2)
            ctx.sync()
        finally:
            ctx.set_option(dci.DCI_OPT_INPUT_LAYER, 0)
            ctx.set_option(dci.DCI_OPT_LINEAR_KERNEL, 0)
        out[kind] = (l1.cpu().numpy()[:len(seeds)], l2.cpu().numpy()[:len(seeds)])
        _logit_check(out[kind][0], ref)
        _logit_check(out[kind][1], ref)
    assert out[3][0].tobytes() == out[3][1].tobytes()
    if hidden % 256 == 0:
        assert out[3][0].tobytes() == out[1][0].tobytes()
        assert out[3][1].tobytes() == out[1][1].tobytes()


def test_gather_forward_rejects_bad_arguments(env):
    dci, gu, ctx, g, tiny, w = (env[k] for k in ("dci", "gu", "ctx", "graph", "tiny", "w"))
    blk = dci.Blocks(ctx, w.num_nodes, 16, w.fanouts)
    dci.dci_sample_khop(ctx, g, None, gu.dev(tiny["seeds"][:16]), 0, w.fanouts, w.rng_seed, blk)
    x = torch.empty(blk.cap_nodes[-1], w.feat_dim, dtype=torch.float32, device="cuda")
    logits = torch.empty(16, 10, dtype=torch.float32, device="cuda")
    ws_h, wn_h, b_h = synth.sage_weights((w.feat_dim + 1, 8, 10), 3)       # wrong input width
    ws, wn, bs = ([gu.dev(a) for a in arr] for arr in (ws_h, wn_h, b_h))
    with pytest.raises(dci.DciError) as e:
        dci.dci_gather_forward(ctx, g, None, blk, x, 0, ws, wn, bs, logits)
    assert e.value.code == -1 and "features" in str(e.value)
