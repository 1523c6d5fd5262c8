"""Pins for the oracle's random numbers, per-node sampler and mini-batch block builder."""
import itertools
import os
from collections import Counter

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _kat_rows():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(x, 16) for x in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers():
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert oracle.philox4x32_10(ctr, key) == want


def test_uniform_below_counter_packing_and_range():
    # key = (seed lo, seed hi); counter = (node lo, node hi, batch, hop << 24 | slot);
    # value = high 64 bits of (x0 | x1 << 32) * m, evaluated here with Python integers.
    cases = [(4, 0, 0, 0, 0, 7), (0x123456789ABCDEF0, (5 << 32) | 17, 1 << 31, 2, 24, 1000003),
             (99, 111_059_955, 7, 255, (1 << 24) - 1, (1 << 63) + 5), (1, 2, 3, 1, 1, 1)]
    for seed, node, batch, hop, slot, m in cases:
        x = oracle.philox4x32_10([node & 0xFFFFFFFF, node >> 32, batch & 0xFFFFFFFF, (hop << 24) | slot],
                                 [seed & 0xFFFFFFFF, seed >> 32])
        want = ((x[0] | (x[1] << 32)) * m) >> 64
        got = oracle.uniform_below(seed, node, batch, hop, slot, m)
        assert got == want and 0 <= got < m


def test_uniform_below_is_uniform():
    m, n = 6, 60000
    counts = Counter(oracle.uniform_below(4, node, 0, 0, 0, m) for node in range(n))
    chi2 = sum((counts[k] - n / m) ** 2 / (n / m) for k in range(m))
    assert chi2 < 25.0  # 5 degrees of freedom: P(chi2 > 25) ~ 1e-4


def test_positions_small_degree_returns_whole_list_in_order():
    for deg in range(0, 8):
        for fanout in range(deg, 10):
            pos = oracle.sample_positions(4, 3, 1, 1234, deg, fanout)
            assert list(pos) == list(range(deg))


def test_positions_are_a_subset_without_replacement():
    for deg, fanout in [(6, 3), (7, 6), (1000, 25), (1 << 40, 15), (16, 15)]:
        for node in range(50):
            pos = oracle.sample_positions(4, 9, 2, node, deg, fanout)
            assert len(pos) == fanout
            assert len(set(pos.tolist())) == fanout
            assert pos.min() >= 0 and pos.max() < deg


def test_floyd_matches_its_definition_from_raw_draws():
    # Rebuild the subset from the raw uniform draws with a Python set; this pins the order of
    # the draws (slot s draws below deg - fanout + s + 1) and the replacement rule.
    for deg, fanout, node in [(6, 3, 5), (40, 10, 77), (9, 8, 3), (100000, 15, 123456)]:
        chosen = []
        for s in range(fanout):
            j = deg - fanout + s
            t = oracle.uniform_below(4, node, 11, 1, s, j + 1)
            chosen.append(j if t in chosen else t)
        assert list(oracle.sample_positions(4, 11, 1, node, deg, fanout)) == chosen


def test_floyd_subsets_equally_likely():
    # degree 6, fan-out 3: the 20 subsets must be equally likely.
    n = 40000
    counts = Counter()
    for node in range(n):
        counts[tuple(sorted(oracle.sample_positions(4, 0, 0, node, 6, 3).tolist()))] += 1
    assert set(counts) == set(itertools.combinations(range(6), 3))
    chi2 = sum((counts[k] - n / 20) ** 2 / (n / 20) for k in counts)
    assert chi2 < 50.0  # 19 degrees of freedom: P(chi2 > 50) ~ 1e-4
    # every position is also equally likely to be chosen first
    first = Counter(int(oracle.sample_positions(4, 0, 0, node, 6, 3)[0]) for node in range(n))
    assert set(first) == set(range(4))  # the first draw is below deg - fanout + 1 = 4


def test_draws_depend_on_every_key_field():
    base = oracle.sample_positions(4, 0, 0, 10, 10**6, 15).tolist()
    assert oracle.sample_positions(5, 0, 0, 10, 10**6, 15).tolist() != base
    assert oracle.sample_positions(4, 1, 0, 10, 10**6, 15).tolist() != base
    assert oracle.sample_positions(4, 0, 1, 10, 10**6, 15).tolist() != base
    assert oracle.sample_positions(4, 0, 0, 11, 10**6, 15).tolist() != base
    assert oracle.sample_positions(4, 0, 0, 10, 10**6, 15).tolist() == base


def _check_blocks(indptr, indices, seeds, fanouts, blk, batch_index, rng_seed):
    L = len(fanouts)
    assert blk.n_nodes[0] == len(seeds)
    assert list(blk.nodes[:len(seeds)]) == list(seeds)
    assert len(set(blk.nodes.tolist())) == len(blk.nodes)      # F_L has no duplicates
    local = {int(v): i for i, v in enumerate(seeds)}
    frontier = [int(v) for v in seeds]
    for h in range(L):
        n_h = int(blk.n_nodes[h])
        assert len(blk.blk_indptr[h]) == n_h + 1 and blk.blk_indptr[h][0] == 0
        assert blk.blk_indptr[h][-1] == blk.n_edges[h] == len(blk.blk_src[h])
        for i in range(n_h):
            v = int(blk.nodes[i])
            deg = int(indptr[v + 1] - indptr[v])
            e0, e1 = int(blk.blk_indptr[h][i]), int(blk.blk_indptr[h][i + 1])
            assert e1 - e0 == min(fanouts[h], deg)                      # fan-out and degree caps
            pos = blk.src_pos[h][e0:e1]
            assert len(set(pos.tolist())) == e1 - e0                     # without replacement
            for e in range(e0, e1):
                assert 0 <= pos[e - e0] < deg
                u = int(indices[indptr[v] + pos[e - e0]])                # the edge exists, at that position
                assert u == int(blk.src_global[h][e])
                if u not in local:                                       # first appearance order
                    local[u] = len(frontier)
                    frontier.append(u)
                assert local[u] == int(blk.blk_src[h][e])
            if deg <= fanouts[h]:
                assert pos.tolist() == list(range(deg))                  # verbatim list
            else:
                assert pos.tolist() == oracle.sample_positions(rng_seed, batch_index, h, v, deg, fanouts[h]).tolist()
        assert blk.n_nodes[h + 1] == len(frontier)
        assert blk.nodes[:len(frontier)].tolist() == frontier           # F_h is a prefix of F_{h+1}


def test_blocks_brute_force_small_graphs(small_graphs):
    for gi, (indptr, indices) in enumerate(small_graphs):
        n = len(indptr) - 1
        rng = np.random.default_rng(gi)
        for fanouts in [(2,), (3, 2), (2, 2, 2), (1, 4, 3), (64, 1)]:
            seeds = rng.permutation(n)[:max(1, n // 4)].astype(np.int64)
            blk = oracle.sample_khop(indptr, indices, seeds, 5 + gi, fanouts, 4)
            _check_blocks(indptr, indices, seeds, fanouts, blk, 5 + gi, 4)


def test_blocks_tiny_workload(tiny):
    w = tiny["w"]
    seeds = tiny["seeds"][:w.batch_size]
    blk = oracle.sample_khop(tiny["indptr"], tiny["indices"], seeds, 0, w.fanouts, w.rng_seed)
    _check_blocks(tiny["indptr"], tiny["indices"], seeds, w.fanouts, blk, 0, w.rng_seed)
    caps = w.cap_nodes()
    assert all(blk.n_nodes[h] <= caps[h] for h in range(len(caps)))


def test_empty_and_degenerate_batches(small_graphs):
    indptr, indices = small_graphs[3]
    blk = oracle.sample_khop(indptr, indices, np.array([], dtype=np.int64), 0, (2, 2), 4)
    assert blk.n_nodes.tolist() == [0, 0, 0] and blk.n_edges.tolist() == [0, 0]
    # seeds without in-neighbours give empty rows and no growth
    blk = oracle.sample_khop(indptr, indices, np.array([0, 4], dtype=np.int64), 0, (2, 2), 4)
    assert blk.n_nodes.tolist() == [2, 2, 2] and blk.n_edges.tolist() == [0, 0]
    assert blk.blk_indptr[0].tolist() == [0, 0, 0]
    # duplicated neighbours in a multigraph list are separate positions with one local id
    blk = oracle.sample_khop(indptr, indices, np.array([1], dtype=np.int64), 0, (3,), 4)
    assert blk.src_global[0].tolist() == [1, 3, 3]
    assert blk.blk_src[0].tolist() == [0, 1, 1] and blk.nodes.tolist() == [1, 3]


def test_batches_are_independent_of_processing_order(tiny):
    w = tiny["w"]
    args = (tiny["indptr"], tiny["indices"])
    b0 = oracle.sample_khop(*args, tiny["seeds"][:256], 0, w.fanouts, w.rng_seed)
    b1 = oracle.sample_khop(*args, tiny["seeds"][256:512], 1, w.fanouts, w.rng_seed)
    b1_again = oracle.sample_khop(*args, tiny["seeds"][256:512], 1, w.fanouts, w.rng_seed)
    b0_again = oracle.sample_khop(*args, tiny["seeds"][:256], 0, w.fanouts, w.rng_seed)
    for x, y in [(b0, b0_again), (b1, b1_again)]:
        assert x.nodes.tolist() == y.nodes.tolist()
        for h in range(w.n_hops):
            assert x.blk_src[h].tolist() == y.blk_src[h].tolist()
