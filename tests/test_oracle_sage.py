"""Pins for the oracle's GraphSAGE-mean forward pass."""
import numpy as np

import oracle


def _dense_forward(blk, x, w_self, w_neigh, bias, model=0):
    """Independent formulation: per layer build the sampled adjacency A_s as a dense matrix and use
    matrix products (numpy, fp64): D^-1 A_s for the mean, A_s for the sum, (D+I)^-1 (A_s + I) for GCN."""
    L = len(w_neigh)
    x = x.astype(np.float64)
    for l in range(L):
        h = L - 1 - l
        n_dst, n_src = int(blk.n_nodes[h]), int(blk.n_nodes[h + 1])
        A = np.zeros((n_dst, n_src))
        rows = np.repeat(np.arange(n_dst), np.diff(blk.blk_indptr[h]))
        np.add.at(A, (rows, blk.blk_src[h]), 1.0)
        if model == 2:
            A[np.arange(n_dst), np.arange(n_dst)] += 1.0
        if model != 1:
            d = A.sum(axis=1, keepdims=True)
            A = np.divide(A, d, out=np.zeros_like(A), where=d > 0)
        y = (A @ x[:n_src]) @ w_neigh[l].astype(np.float64) + bias[l]
        if model != 2:
            y = y + x[:n_dst] @ w_self[l].astype(np.float64)
        x = np.maximum(y, 0.0) if l != L - 1 else y
    return x


def test_sum_and_gcn_variants_match_dense_formulation(tiny, small_graphs):
    w = tiny["w"]
    blk = oracle.sample_khop(tiny["indptr"], tiny["indices"], tiny["seeds"][:64], 0, w.fanouts, w.rng_seed)
    x = tiny["feat"][blk.nodes]
    outs = {}
    for model in (oracle.SAGE_MEAN, oracle.SAGE_SUM, oracle.GCN_AVG):
        got = oracle.gnn_forward(model, blk, x, tiny["w_self"], tiny["w_neigh"], tiny["bias"])
        want = _dense_forward(blk, x, tiny["w_self"], tiny["w_neigh"], tiny["bias"], model)
        assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
        outs[model] = got
    assert not np.allclose(outs[0], outs[1]) and not np.allclose(outs[0], outs[2])
    # empty rows: sum gives zero, GCN gives the node's own features
    indptr, indices = small_graphs[3]
    blk = oracle.sample_khop(indptr, indices, np.array([0, 4, 1], dtype=np.int64), 1, (2,), 4)
    xx = np.arange(len(blk.nodes) * 3, dtype=np.float32).reshape(-1, 3) + 1
    eye, zero, b0 = np.eye(3, dtype=np.float32), np.zeros((3, 3), dtype=np.float32), np.zeros(3, dtype=np.float32)
    got = oracle.gnn_forward(oracle.GCN_AVG, blk, xx, None, [eye], [b0])
    assert np.array_equal(got[:2], xx[:2].astype(np.float64))           # nodes 0 and 4 have no in-neighbours
    got = oracle.gnn_forward(oracle.SAGE_SUM, blk, xx, [zero], [eye], [b0])
    assert np.array_equal(got[:2], np.zeros((2, 3)))
    e0, e1 = blk.blk_indptr[0][2], blk.blk_indptr[0][3]
    assert np.allclose(got[2], xx[blk.blk_src[0][e0:e1]].astype(np.float64).sum(axis=0))


def test_matches_dense_formulation(tiny):
    w = tiny["w"]
    blk = oracle.sample_khop(tiny["indptr"], tiny["indices"], tiny["seeds"][:64], 0, w.fanouts, w.rng_seed)
    x = tiny["feat"][blk.nodes]
    got = oracle.sage_forward(blk, x, tiny["w_self"], tiny["w_neigh"], tiny["bias"])
    want = _dense_forward(blk, x, tiny["w_self"], tiny["w_neigh"], tiny["bias"])
    assert got.shape == (64, w.classes)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    assert np.abs(got).max() > 0.1


def test_three_layers_with_empty_rows(small_graphs):
    indptr, indices = small_graphs[3]              # has nodes without in-neighbours
    rng = np.random.default_rng(5)
    seeds = np.array([0, 1, 3, 4], dtype=np.int64)
    blk = oracle.sample_khop(indptr, indices, seeds, 1, (2, 2, 2), 4)
    dims = [6, 5, 4, 3]
    x = rng.standard_normal((len(blk.nodes), dims[0])).astype(np.float32)
    ws = [rng.standard_normal((dims[i], dims[i + 1])).astype(np.float32) for i in range(3)]
    wn = [rng.standard_normal((dims[i], dims[i + 1])).astype(np.float32) for i in range(3)]
    bs = [rng.standard_normal(dims[i + 1]).astype(np.float32) for i in range(3)]
    got = oracle.sage_forward(blk, x, ws, wn, bs)
    assert np.allclose(got, _dense_forward(blk, x, ws, wn, bs), rtol=1e-12, atol=1e-12)


def test_identity_self_weight_returns_input_rows(tiny):
    w = tiny["w"]
    blk = oracle.sample_khop(tiny["indptr"], tiny["indices"], tiny["seeds"][:32], 0, (5,), w.rng_seed)
    x = tiny["feat"][blk.nodes]
    F = w.feat_dim
    got = oracle.sage_forward(blk, x, [np.eye(F, dtype=np.float32)], [np.zeros((F, F), dtype=np.float32)],
                              [np.zeros(F, dtype=np.float32)])
    assert np.array_equal(got, x[:32].astype(np.float64))      # no ReLU after the last layer
    # identity on the neighbour side instead: logits are the sampled neighbours' mean
    got = oracle.sage_forward(blk, x, [np.zeros((F, F), dtype=np.float32)], [np.eye(F, dtype=np.float32)],
                              [np.zeros(F, dtype=np.float32)])
    for i in range(32):
        e0, e1 = blk.blk_indptr[0][i], blk.blk_indptr[0][i + 1]
        want = x[blk.blk_src[0][e0:e1]].astype(np.float64).mean(axis=0) if e1 > e0 else np.zeros(F)
        assert np.allclose(got[i], want, rtol=1e-13, atol=1e-13)


def test_all_ones_features(tiny):
    w = tiny["w"]
    blk = oracle.sample_khop(tiny["indptr"], tiny["indices"], tiny["seeds"][:32], 0, (5,), w.rng_seed)
    x = np.ones((len(blk.nodes), w.feat_dim), dtype=np.float32)
    ws, wn, b = tiny["w_self"][0], tiny["w_neigh"][0], tiny["bias"][0]
    got = oracle.sage_forward(blk, x, [ws], [wn], [b])
    has = np.diff(blk.blk_indptr[0]) > 0
    want_full = ws.astype(np.float64).sum(0) + wn.astype(np.float64).sum(0) + b
    want_empty = ws.astype(np.float64).sum(0) + b
    assert has.any()
    assert np.allclose(got[has], want_full, rtol=1e-12)
    if (~has).any():
        assert np.allclose(got[~has], want_empty, rtol=1e-12)


def test_relu_between_layers_only():
    # one destination, one neighbour; weights chosen so the hidden value is negative
    from oracle import Blocks
    blk = Blocks(n_nodes=np.array([1, 1, 2]), n_edges=np.array([0, 1]), nodes=np.array([0, 1]),
                 blk_indptr=[np.array([0, 0]), np.array([0, 1])], blk_src=[np.array([], dtype=np.int32),
                                                                          np.array([1], dtype=np.int32)],
                 src_global=[], src_pos=[])
    x = np.array([[1.0], [3.0]], dtype=np.float32)
    one, neg, zero = (np.array([[v]], dtype=np.float32) for v in (1.0, -1.0, 0.0))
    b0 = np.zeros(1, dtype=np.float32)
    # layer 0 on block 1: y = 1*(-1) + 3*(-1) = -4 -> ReLU -> 0 ; layer 1 on block 0: 0*1 + 0 - 2 = -2 (kept)
    got = oracle.sage_forward(blk, x, [neg, one], [neg, zero], [b0, np.array([-2.0], dtype=np.float32)])
    assert got.tolist() == [[-2.0]]


def test_run_batches_is_the_three_calls_per_batch_whatever_the_thread_count(tiny):
    """The multi-thread driver used for the benchmark's all-cores figure adds no arithmetic of its own:
    totals and the sum of all logits equal those of sample_khop -> gather -> gnn_forward called batch by
    batch, for 1, 3 and 8 threads, including a ragged last batch and a range that runs past the end."""
    w = tiny["w"]
    B = 200                                            # 2,048 seeds -> 10 full batches and one of 48
    edges = rows = 0
    total = 0.0
    for b in range(3, 11):
        s = tiny["seeds"][b * B:(b + 1) * B]
        blk = oracle.sample_khop(tiny["indptr"], tiny["indices"], s, b, w.fanouts, w.rng_seed)
        x = oracle.gather(tiny["feat"], blk.nodes)
        total += float(oracle.gnn_forward(1, blk, x, tiny["w_self"], tiny["w_neigh"], tiny["bias"]).sum())
        edges += int(blk.n_edges.sum())
        rows += len(blk.nodes)
    for threads in (1, 3, 8):
        r = oracle.run_batches(tiny["indptr"], tiny["indices"], tiny["feat"], tiny["seeds"], B, 3, 50, w.fanouts,
                               w.rng_seed, 1, tiny["w_self"], tiny["w_neigh"], tiny["bias"], n_threads=threads)
        assert (r["edges"], r["input_rows"], r["batches"]) == (edges, rows, 8)
        assert abs(r["logit_sum"] - total) <= 1e-9 * max(1.0, abs(total))
        assert r["wall_s"] > 0 and r["sample_s"] > 0 and r["forward_s"] > 0
