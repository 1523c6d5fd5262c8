"""Pins for pre-sampling counts, the capacity split and the two cache fills of the oracle."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------------------ counting

def _tally(indptr, indices, seeds, batch_size, n_batches, fanouts, rng_seed, rng_batch0):
    """Explicit tallies from the emitted blocks, with dictionaries."""
    feat, adj, edge = {}, {}, {}
    edges = nodes = 0
    for b in range(n_batches):
        s = seeds[b * batch_size:(b + 1) * batch_size]
        if len(s) == 0:
            break
        blk = oracle.sample_khop(indptr, indices, s, rng_batch0 + b, fanouts, rng_seed)
        for h in range(len(fanouts)):
            for i in range(int(blk.n_nodes[h])):
                v = int(blk.nodes[i])
                for e in range(int(blk.blk_indptr[h][i]), int(blk.blk_indptr[h][i + 1])):
                    adj[v] = adj.get(v, 0) + 1
                    k = int(indptr[v] + blk.src_pos[h][e])
                    edge[k] = edge.get(k, 0) + 1
                    edges += 1
        for u in blk.nodes.tolist():
            feat[u] = feat.get(u, 0) + 1
            nodes += 1
    return feat, adj, edge, edges, nodes


def _dense(d, n):
    out = np.zeros(n, dtype=np.uint32)
    for k, v in d.items():
        out[k] = v
    return out


def test_counts_equal_explicit_tallies(small_graphs):
    for indptr, indices in small_graphs:
        n = len(indptr) - 1
        seeds = np.random.default_rng(1).permutation(n)[:max(2, n // 2)].astype(np.int64)
        for fanouts, bs in [((2, 3), 7), ((3,), 4), ((2, 2, 2), 1000)]:
            nb = 3
            fc, ac, ec, (edges, nodes) = oracle.presample_count(indptr, indices, seeds, bs, nb, fanouts, 4, 1 << 31)
            feat, adj, edge, e_want, n_want = _tally(indptr, indices, seeds, bs, nb, fanouts, 4, 1 << 31)
            assert np.array_equal(fc, _dense(feat, n))
            assert np.array_equal(ac, _dense(adj, n))
            assert np.array_equal(ec, _dense(edge, len(indices)))
            assert (edges, nodes) == (e_want, n_want)


def test_count_invariants_tiny(tiny):
    w = tiny["w"]
    indptr, indices = tiny["indptr"], tiny["indices"]
    fc, ac, ec, (edges, nodes) = oracle.presample_count(indptr, indices, tiny["seeds"], w.batch_size,
                                                        w.n_presample, w.fanouts, w.rng_seed,
                                                        w.presample_first_batch)
    # per-node totals are the sums of the per-element counts of the node's list
    per_node = np.add.reduceat(np.concatenate([ec, [0]]).astype(np.int64), indptr[:-1])
    per_node[np.diff(indptr) == 0] = 0
    assert np.array_equal(per_node, ac.astype(np.int64))
    assert int(ac.sum()) == edges and int(fc.sum()) == nodes
    assert fc.max() <= w.n_presample  # a node is visited at most once per batch
    # accumulation: two calls over half the batches each equal one call over all
    fc2, ac2, ec2, _ = oracle.presample_count(indptr, indices, tiny["seeds"], w.batch_size, 4, w.fanouts,
                                              w.rng_seed, w.presample_first_batch)
    oracle.presample_count(indptr, indices, tiny["seeds"], w.batch_size, 4, w.fanouts, w.rng_seed,
                           w.presample_first_batch + 4, first_batch=4, feat_count=fc2, adj_count=ac2,
                           edge_count=ec2)
    assert np.array_equal(fc, fc2) and np.array_equal(ac, ac2) and np.array_equal(ec, ec2)


# ------------------------------------------------------------------------------ Eq. (1)

def test_split_closed_form():
    # 3:7 on C = 1000 with both sides far larger than their share
    assert oracle.split(1000, 3, 7, 1000, 10000, 64) == (300, 700)
    assert oracle.split(1000, 7, 3, 1000, 10000, 64) == (700, 300)
    assert oracle.split(1000, 0, 0, 1000, 10000, 64) == (500, 500)
    assert oracle.split(1000, 5, 0, 1000, 10000, 64) == (1000, 0)
    assert oracle.split(1001, 1, 2, 1000, 10000, 64) == (333, 668)      # floor on the adjacency side
    for C, ts, tf in [(123456789, 17, 5), (2**45 + 1, 2**63, 2**62 + 3), (10, 1, 1)]:   # needs 128-bit products
        a, f = oracle.split(C, ts, tf, 10**12, 10**13, 128)
        assert a + f == C and a == (C * ts) // (ts + tf)


def test_split_spill_over():
    N, E, F = 10, 30, 4
    A, Ft = (N + 1 + E) * 8, N * F * 4           # 328, 160
    # adjacency share exceeds the whole structure: the excess goes to features
    assert oracle.split(1000, 9, 1, N, E, F) == (A, 1000 - A)
    # feature share exceeds the whole matrix: the excess goes to the adjacency side
    assert oracle.split(400, 1, 9, N, E, F) == (400 - Ft, Ft)
    # a budget that covers the whole dataset caches all of it, whatever the time ratio
    for ts, tf in [(1, 99), (99, 1), (1, 1), (0, 0)]:
        a, f = oracle.split(A + Ft, ts, tf, N, E, F)
        assert a >= A and f >= Ft
    # without spill-over the shares of Eq. (1) stand; t_sample = 0 is the single-cache system
    assert oracle.split(1000, 9, 1, N, E, F, spill=False) == (900, 100)
    assert oracle.split(400, 1, 9, N, E, F, spill=False) == (40, 360)
    assert oracle.split(400, 0, 5, N, E, F, spill=False) == (0, 400)


# ------------------------------------------------------------------------------ feature fill

def test_feature_fill_policies_against_numpy(tiny):
    w = tiny["w"]
    fc, _, _, _ = oracle.presample_count(tiny["indptr"], tiny["indices"], tiny["seeds"], w.batch_size,
                                         w.n_presample, w.fanouts, w.rng_seed, w.presample_first_batch,
                                         with_edge_count=False)
    N, F = w.num_nodes, w.feat_dim
    ids = np.arange(N)
    above = fc.astype(np.int64) * N > int(fc.sum())
    assert 0 < above.sum() < N
    for k_want in [0, 1, int(above.sum()) - 3, int(above.sum()), int(above.sum()) + 100, N, N + 5]:
        C_feat = k_want * 4 * F + 17
        k = min(N, k_want)
        # the paper's rule: above-mean nodes first (id order), then the rest (id order)
        remap, cache, got_k = oracle.fill_feat(fc, tiny["feat"], C_feat, 0)
        order = np.lexsort((ids, ~above))
        want = np.full(N, -1, dtype=np.int32)
        want[order[:k]] = np.arange(k, dtype=np.int32)
        assert got_k == k and np.array_equal(remap, want)
        assert np.array_equal(cache, tiny["feat"][order[:k]])
        if k >= above.sum():
            assert (remap[above] >= 0).all()            # every above-mean node is cached
        # top-k by count, ties by id
        remap1, cache1, _ = oracle.fill_feat(fc, tiny["feat"], C_feat, 1)
        order1 = np.lexsort((ids, -fc.astype(np.int64)))
        want1 = np.full(N, -1, dtype=np.int32)
        want1[order1[:k]] = np.arange(k, dtype=np.int32)
        assert np.array_equal(remap1, want1) and np.array_equal(cache1, tiny["feat"][order1[:k]])


def test_feature_fill_mean_is_over_all_nodes():
    # counts 0,0,0,4: mean over all four nodes is 1, so only node 3 is above it; node ids then fill in order
    fc = np.array([0, 0, 0, 4], dtype=np.uint32)
    remap, _, k = oracle.fill_feat(fc, None, 3 * 8, 0, feat_dim=2)
    assert k == 3 and remap.tolist() == [1, 2, -1, 0]
    # a count equal to the mean is not "greater than the average"
    fc = np.array([1, 1, 1, 1], dtype=np.uint32)
    remap, _, _ = oracle.fill_feat(fc, None, 2 * 8, 0, feat_dim=2)
    assert remap.tolist() == [0, 1, -1, -1]
    # counts 1,0,2,1 (mean 1): only node 2 is above; nodes 0 and 3 sit exactly on the mean and follow in id order
    fc = np.array([1, 0, 2, 1], dtype=np.uint32)
    remap, _, _ = oracle.fill_feat(fc, None, 2 * 8, 0, feat_dim=2)
    assert remap.tolist() == [1, -1, 0, -1]


# ------------------------------------------------------------------------------ adjacency fill

def _read_toy():
    lists, counts = {}, {}
    with open(os.path.join(GOLDEN, "fig6_toy.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            node, rest = line.split(":")
            items = [t for t in rest.split()]
            lists[int(node)] = [int(t.split("(")[0]) for t in items]
            counts[int(node)] = [int(t.split("(")[1].rstrip(")")) for t in items]
    n = 8
    indptr = np.zeros(n + 1, dtype=np.int64)
    for v in range(n):
        indptr[v + 1] = indptr[v] + len(lists.get(v, []))
    indices = np.array([u for v in range(n) for u in lists.get(v, [])], dtype=np.int64)
    edge_count = np.array([c for v in range(n) for c in counts.get(v, [])], dtype=np.uint32)
    return indptr, indices, edge_count


def test_adjacency_fill_worked_example():
    indptr, indices, edge_count = _read_toy()
    n = len(indptr) - 1
    node_totals = np.array([edge_count[indptr[v]:indptr[v + 1]].sum() for v in range(n)], dtype=np.uint32)
    assert node_totals[0] == 22 and node_totals[1] == 12          # the sums the paper states
    # room for nodes 0 and 3 and 1 only: 8 + (3+1)*8 + (2+1)*8 + (2+1)*8 = 88 bytes
    remap, cp, ci = oracle.fill_adj(indptr, indices, node_totals, 88)
    assert remap.tolist() == [0, 2, -1, 1, -1, -1, -1, -1]        # node 0 before node 3 before node 1
    assert cp.tolist() == [0, 3, 5, 7] and ci.tolist() == [4, 6, 7, 1, 2, 2, 5]
    # one byte less and node 1 no longer fits; the slice stops there (no skipping to later nodes)
    remap, cp, ci = oracle.fill_adj(indptr, indices, node_totals, 87)
    assert remap.tolist() == [0, -1, -1, 1, -1, -1, -1, -1]
    # the whole structure fits: cached verbatim, slot = node id
    remap, cp, ci = oracle.fill_adj(indptr, indices, node_totals, (n + 1 + len(indices)) * 8)
    assert remap.tolist() == list(range(n)) and np.array_equal(cp, indptr) and np.array_equal(ci, indices)
    # one byte short of the whole structure: the sorted, sliced branch
    remap, cp, ci = oracle.fill_adj(indptr, indices, node_totals, (n + 1 + len(indices)) * 8 - 1)
    assert remap.tolist() == [0, 2, 3, 1, 4, 5, 6, -1]


def test_adjacency_fill_against_numpy(tiny):
    w = tiny["w"]
    indptr, indices = tiny["indptr"], tiny["indices"]
    _, ac, _, _ = oracle.presample_count(indptr, indices, tiny["seeds"], w.batch_size, w.n_presample, w.fanouts,
                                         w.rng_seed, w.presample_first_batch, with_edge_count=False)
    N = w.num_nodes
    deg = np.diff(indptr)
    order = np.argsort(-ac.astype(np.int64), kind="stable")
    cum = 8 + np.cumsum(8 * deg[order] + 8)
    for C_adj in [0, 7, 8, 16, 5000, 123457, 600000, w.adj_bytes - 1]:
        K = int(np.searchsorted(cum, C_adj, side="right"))
        remap, cp, ci = oracle.fill_adj(indptr, indices, ac, C_adj)
        want = np.full(N, -1, dtype=np.int32)
        want[order[:K]] = np.arange(K, dtype=np.int32)
        assert np.array_equal(remap, want)
        assert len(cp) == K + 1 and np.array_equal(np.diff(cp), deg[order[:K]])
        used = 8 * (K + 1) + 8 * len(ci)
        assert used <= max(C_adj, 8)
        if K < N:
            assert used + 8 * deg[order[K]] + 8 > C_adj       # the next node would not fit
        # hit = miss: every cached list holds the bytes of the host list, in the host order
        for s in np.random.default_rng(0).permutation(K)[:200]:
            v = order[s]
            assert np.array_equal(ci[cp[s]:cp[s + 1]], indices[indptr[v]:indptr[v + 1]])
    remap, cp, ci = oracle.fill_adj(indptr, indices, ac, w.adj_bytes)
    assert np.array_equal(remap, np.arange(N)) and np.array_equal(cp, indptr) and np.array_equal(ci, indices)


# ------------------------------------------------------------------------------ cache transparency

def test_cached_routes_return_identical_results(tiny):
    w = tiny["w"]
    indptr, indices, feat = tiny["indptr"], tiny["indices"], tiny["feat"]
    fc, ac, _, _ = oracle.presample_count(indptr, indices, tiny["seeds"], w.batch_size, w.n_presample, w.fanouts,
                                          w.rng_seed, w.presample_first_batch, with_edge_count=False)
    C_adj, C_feat = oracle.split(w.budget_bytes, 3, 7, w.num_nodes, w.num_edges, w.feat_dim)
    assert C_adj + C_feat == w.budget_bytes
    adj_remap, cp, ci = oracle.fill_adj(indptr, indices, ac, C_adj)
    feat_remap, fcache, k = oracle.fill_feat(fc, feat, C_feat, 0)
    assert 0 < (adj_remap >= 0).sum() < w.num_nodes and 0 < k < w.num_nodes
    seeds = tiny["seeds"][512:768]
    blk = oracle.sample_khop(indptr, indices, seeds, 2, w.fanouts, w.rng_seed)
    for h in range(w.n_hops):
        frontier = blk.nodes[:blk.n_nodes[h]]
        rows, src, counts = oracle.sample_hop_cached(indptr, indices, adj_remap, cp, ci, frontier, 2, h,
                                                     w.fanouts[h], w.rng_seed)
        assert np.array_equal(rows, np.diff(blk.blk_indptr[h]))
        assert np.array_equal(src, blk.src_global[h])
        hit = adj_remap[frontier] >= 0
        assert counts.tolist() == [hit.sum(), (~hit).sum(), rows[hit].sum(), rows[~hit].sum()]
        assert counts[0] > 0 and counts[1] > 0
    rows, hits, misses = oracle.gather_cached(feat, feat_remap, fcache, blk.nodes)
    plain = oracle.gather(feat, blk.nodes)
    assert rows.tobytes() == plain.tobytes() == feat[blk.nodes].tobytes()
    assert hits == (feat_remap[blk.nodes] >= 0).sum() and hits > 0 and misses > 0


# ---- element-granular adjacency cache (Algorithm 1 / Fig. 6 as printed) --------------------------------------

def test_element_fill_worked_example():
    """Fig. 6 narrative: node 0 (22 visits) before node 1 (12); node 0's elements 4, 6, 7 reorder to 7, 6, 4;
    node 2 has two elements of which one is cached; position n of node 2 hits iff n <= 1 (1-based)."""
    indptr, indices, edge_count = _read_toy()
    # nodes 0, 3, 1 whole (88 bytes, see above) + node 2's pointer entry and one element (16 bytes)
    remap, cp, ci, idx, pn, pd = oracle.fill_adj_element(indptr, indices, edge_count, 104)
    assert remap.tolist() == [0, 2, 3, 1, -1, -1, -1, -1]
    assert idx.tolist() == [7, 6, 4, 2, 5, 0, 3, 1, 2]             # every node reordered by element count
    assert cp.tolist() == [0, 3, 5, 7, 8] and ci.tolist() == [7, 6, 4, 1, 2, 2, 5, 0]
    assert (pn, pd) == (2, 2)
    # the hit rule on node 2: a fan-out of 2 takes both positions; the first is served by the cache
    rows, src, counts = oracle.sample_hop_cached(indptr, idx, remap, cp, ci, np.array([2]), 0, 0, 2, 1, pn, pd)
    assert rows.tolist() == [2] and src.tolist() == [0, 3] and counts.tolist() == [1, 0, 1, 1]
    # one byte less: no room for pointer entry + element of node 2 (needs 16), the slice ends with node 1
    remap, cp, ci, idx, pn, pd = oracle.fill_adj_element(indptr, indices, edge_count, 103)
    assert remap.tolist() == [0, 2, -1, 1, -1, -1, -1, -1] and cp.tolist() == [0, 3, 5, 7] and (pn, pd) == (-1, 0)
    # 8 bytes short of node 1 as a whole: node 1 becomes the partial node with one of its two elements
    remap, cp, ci, idx, pn, pd = oracle.fill_adj_element(indptr, indices, edge_count, 80)
    assert remap.tolist() == [0, 2, -1, 1, -1, -1, -1, -1] and cp.tolist() == [0, 3, 5, 6] and ci.tolist()[-1] == 2
    assert (pn, pd) == (1, 2)
    # the whole structure fits: verbatim, nothing reordered
    n = len(indptr) - 1
    remap, cp, ci, idx, pn, pd = oracle.fill_adj_element(indptr, indices, edge_count, (n + 1 + len(indices)) * 8)
    assert remap.tolist() == list(range(n)) and np.array_equal(ci, indices) and np.array_equal(idx, indices) and pn == -1


def _element_fill_by_hand(indptr, indices, edge_count, C_adj):
    """Independent restatement with Python lists and sorted()."""
    n = len(indptr) - 1
    lists = [list(indices[indptr[v]:indptr[v + 1]]) for v in range(n)]
    cnts = [list(edge_count[indptr[v]:indptr[v + 1]]) for v in range(n)]
    if (n + 1 + len(indices)) * 8 <= C_adj:
        return list(range(n)), lists, [len(l) for l in lists], lists
    totals = [sum(int(c) for c in cs) for cs in cnts]
    order = sorted(range(n), key=lambda v: (-totals[v], v))
    new_lists = []
    for v in range(n):
        perm = sorted(range(len(lists[v])), key=lambda t: (-int(cnts[v][t]), t))
        new_lists.append([lists[v][t] for t in perm])
    stream_budget = C_adj - 8
    slots, lens = [], []
    for v in order:
        need = 8 + 8 * len(new_lists[v])
        if stream_budget >= need:
            slots.append(v); lens.append(len(new_lists[v])); stream_budget -= need
        else:
            if stream_budget >= 16:
                slots.append(v); lens.append((stream_budget - 8) // 8)
            break
    if C_adj < 8:
        slots, lens = [], []
    return slots, [new_lists[v][:l] for v, l in zip(slots, lens)], lens, new_lists


def test_element_fill_against_restatement(small_graphs):
    rng = np.random.default_rng(21)
    for indptr, indices in small_graphs:
        n, e = len(indptr) - 1, len(indices)
        for trial in range(6):
            edge_count = (rng.integers(0, 4, e) * rng.integers(0, 2, e)).astype(np.uint32)   # many zeros and ties
            for C_adj in [0, 7, 8, 24, 8 * (n // 2), 8 * (e // 3) + 4, 8 * e, (n + 1 + e) * 8 - 1, (n + 1 + e) * 8]:
                remap, cp, ci, idx, pn, pd = oracle.fill_adj_element(indptr, indices, edge_count, C_adj)
                slots, cached, lens, new_lists = _element_fill_by_hand(indptr, indices, edge_count, C_adj)
                want_remap = -np.ones(n, dtype=np.int64)
                for s, v in enumerate(slots):
                    want_remap[v] = s
                assert np.array_equal(remap, want_remap)
                assert np.array_equal(np.diff(cp), lens) and ci.tolist() == [u for l in cached for u in l]
                assert idx.tolist() == [u for l in new_lists for u in l]
                partial = [v for v, l in zip(slots, lens) if l < indptr[v + 1] - indptr[v]]
                assert ([pn] if pn >= 0 else []) == partial
                if pn >= 0:
                    assert pd == indptr[pn + 1] - indptr[pn]
                # the budget is respected and used to the last whole element
                used = 8 * (len(slots) + 1) + 8 * len(ci) if C_adj >= 8 else 0
                assert used <= max(C_adj, 0)


def test_element_fill_reduces_to_node_fill_when_counts_are_flat(tiny):
    """With the same count on every element of a node the in-node order is unchanged; on a budget that ends at a
    node boundary the element-granular cache is the node-granular one."""
    indptr, indices = tiny["indptr"], tiny["indices"]
    n = len(indptr) - 1
    rng = np.random.default_rng(5)
    per_node = rng.integers(0, 5, n).astype(np.uint32)
    deg = np.diff(indptr)
    edge_count = np.repeat(per_node, deg)
    totals = (per_node.astype(np.uint64) * deg.astype(np.uint64)).astype(np.uint32)
    remap0, cp0, ci0 = oracle.fill_adj(indptr, indices, totals, 200_000)
    boundary = 8 * (len(cp0) + len(ci0))                      # bytes used by the node-granular cache
    remap, cp, ci, idx, pn, pd = oracle.fill_adj_element(indptr, indices, edge_count, boundary + 15)
    assert pn == -1 and np.array_equal(idx, indices)
    assert np.array_equal(remap, remap0) and np.array_equal(cp, cp0) and np.array_equal(ci, ci0)
    # sixteen more bytes buy the pointer entry and the first element of the next node
    remap, cp, ci, idx, pn, pd = oracle.fill_adj_element(indptr, indices, edge_count, boundary + 16)
    assert pn >= 0 and remap[pn] == len(cp0) - 1 and len(ci) == len(ci0) + 1 and ci[-1] == indices[indptr[pn]]


def test_element_cache_is_transparent_to_sampling(tiny):
    """Hit and miss paths return the same bytes: sampling through the element-granular cache equals sampling
    the reordered host structure without a cache, and the hit counters follow the per-position rule."""
    w = tiny["w"]
    indptr, indices = tiny["indptr"], tiny["indices"]
    _, ac, ec, _ = oracle.presample_count(indptr, indices, tiny["seeds"], w.batch_size, w.n_presample, w.fanouts,
                                          w.rng_seed, w.presample_first_batch, with_edge_count=True)
    assert ec.sum() == ac.sum()
    remap, cp, ci, idx, pn, pd = oracle.fill_adj_element(indptr, indices, ec, 300_000 + 8 * 3)
    assert pn >= 0 and 0 < cp[remap[pn] + 1] - cp[remap[pn]] < pd
    # every list is a permutation of the old one, ordered by non-increasing count, ties in the old order
    for v in np.flatnonzero(ac)[:200]:
        s0, s1 = indptr[v], indptr[v + 1]
        perm = sorted(range(s1 - s0), key=lambda t: (-int(ec[s0 + t]), t))
        assert idx[s0:s1].tolist() == indices[s0:s1][perm].tolist()
    seeds = np.concatenate([tiny["seeds"][512:767], [pn]])      # make sure the partial node is sampled
    blk = oracle.sample_khop(indptr, idx, seeds, 2, w.fanouts, w.rng_seed)
    saw_partial_miss = False
    for h in range(w.n_hops):
        frontier = blk.nodes[:blk.n_nodes[h]]
        rows, src, counts = oracle.sample_hop_cached(indptr, idx, remap, cp, ci, frontier, 2, h, w.fanouts[h],
                                                     w.rng_seed, pn, pd)
        assert np.array_equal(rows, np.diff(blk.blk_indptr[h])) and np.array_equal(src, blk.src_global[h])
        slot = remap[frontier]
        clen = np.where(slot >= 0, cp[np.maximum(slot, 0) + 1] - cp[np.maximum(slot, 0)], 0)
        hits = sum(int((blk.src_pos[h][blk.blk_indptr[h][i]:blk.blk_indptr[h][i + 1]] < clen[i]).sum())
                   for i in range(len(frontier)))
        assert counts.tolist() == [(slot >= 0).sum(), (slot < 0).sum(), hits, int(rows.sum()) - hits]
        i_p = np.flatnonzero(frontier == pn)
        if len(i_p):
            p = blk.src_pos[h][blk.blk_indptr[h][i_p[0]]:blk.blk_indptr[h][i_p[0] + 1]]
            saw_partial_miss |= bool((p >= clen[i_p[0]]).any())
    assert saw_partial_miss
