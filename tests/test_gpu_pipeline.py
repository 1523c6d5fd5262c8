"""dci_infer_batches: many batches with several in flight (one lane = context + stream + buffers).

Sixteen consecutive batches of the Tiny workload run on four lanes through partially filled caches (so the
hit and the miss routes of both the sampler and the gather are live), and every batch is compared with the
CPU oracle: blocks and gathered rows bit for bit, logits to 1e-4 of the batch's largest logit.  Blocks and
rows of a batch survive only until its lane takes the next one, so the sixteen batches are run twice: once
in a single call (all logits checked, and the blocks / rows of the last batch of every lane), once four at
a time with every lane's blocks and rows checked in between."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

B = 128          # 2,048 seeds -> 16 batches
N_LANES = 4


@pytest.fixture(scope="module")
def setup(tiny):
    import paper_2503_01281_amd as dci
    from tests import gpu_util as gu
    w = tiny["w"]
    ctx = dci.Context(0)
    g = gu.make_graph(tiny["indptr"], tiny["indices"], tiny["feat"])
    fc, ac, _, _ = oracle.presample_count(tiny["indptr"], tiny["indices"], tiny["seeds"], w.batch_size, w.n_presample,
                                          w.fanouts, w.rng_seed, w.presample_first_batch, with_edge_count=False)
    C_adj, C_feat = oracle.split(w.budget_bytes, 3, 7, w.num_nodes, w.num_edges, w.feat_dim)
    adj_remap, cp, ci = oracle.fill_adj(tiny["indptr"], tiny["indices"], ac, C_adj)
    feat_remap, fcache, k = oracle.fill_feat(fc, tiny["feat"], C_feat, 0)
    assert 0 < (adj_remap >= 0).sum() < w.num_nodes and 0 < k < w.num_nodes      # both caches partial
    cache = gu.upload_cache(adj_remap, cp, ci, feat_remap, fcache)
    weights = [[gu.dev(a) for a in tiny[key]] for key in ("w_self", "w_neigh", "bias")]
    lanes = [dci.Lane(g, B, w.fanouts, w.dims) for _ in range(N_LANES)]
    seeds_dev = gu.dev(tiny["seeds"])
    torch.cuda.synchronize()
    want = []
    for b in range(w.num_seeds // B):
        s = tiny["seeds"][b * B:(b + 1) * B]
        blk = oracle.sample_khop(tiny["indptr"], tiny["indices"], s, b, w.fanouts, w.rng_seed)
        x = oracle.gather(tiny["feat"], blk.nodes)
        want.append((blk, x))
    return dict(dci=dci, gu=gu, w=w, g=g, cache=cache, weights=weights, lanes=lanes, seeds=seeds_dev, want=want,
                adj_remap=adj_remap, feat_remap=feat_remap, tiny=tiny)


def _check_lane(gu, lane, blk_want, x_want):
    got = gu.blocks_to_host(lane.ctx, lane.blocks)
    gu.assert_blocks_equal(got, blk_want)
    assert lane.x[:len(blk_want.nodes)].cpu().numpy().tobytes() == x_want.tobytes()


def _check_logits(got, ref):
    assert np.abs(got - ref).max() <= 1e-4 * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("model", [0, 2])
def test_sixteen_batches_on_four_lanes(setup, model):
    dci, gu, w, g, cache, lanes, want, tiny = (setup[k] for k in ("dci", "gu", "w", "g", "cache", "lanes", "want", "tiny"))
    ws, wn, bs = setup["weights"]
    nb = len(want)
    assert nb == 16
    ref = [oracle.gnn_forward(model, blk, x, tiny["w_self"], tiny["w_neigh"], tiny["bias"]) for blk, x in want]
    logits = torch.full((w.num_seeds, w.classes), float("nan"), dtype=torch.float32, device="cuda")
    stats = gu.new_stats()
    torch.cuda.synchronize()

    # all sixteen in one call
    dci.dci_infer_batches(lanes, g, cache, setup["seeds"], B, 0, nb, w.fanouts, w.rng_seed, model,
                          None if model == 2 else ws, wn, bs, logits, stats)
    for ln in lanes:
        ln.ctx.sync()
    out = logits.cpu().numpy()
    for b in range(nb):
        _check_logits(out[b * B:(b + 1) * B], ref[b])
    for k, ln in enumerate(lanes):                       # lane k ran batches k, k+4, k+8, k+12
        _check_lane(gu, ln, *want[nb - N_LANES + k])
    st = {k: int(v) for k, v in zip(dci.STAT.keys(), stats.cpu().numpy())}
    assert st["edges_sampled"] == sum(int(blk.n_edges.sum()) for blk, _ in want)
    assert st["input_nodes"] == sum(len(blk.nodes) for blk, _ in want)
    hits = sum(int((setup["feat_remap"][blk.nodes] >= 0).sum()) for blk, _ in want)
    assert (st["feat_hits"], st["feat_misses"]) == (hits, st["input_nodes"] - hits)
    assert 0 < st["adj_edge_hits"] < st["edges_sampled"] and 0 < hits < st["input_nodes"]

    # four at a time, every lane's blocks and rows checked while they are still there
    logits.fill_(float("nan"))
    for first in range(0, nb, N_LANES):
        dci.dci_infer_batches(lanes, g, cache, setup["seeds"], B, first, N_LANES, w.fanouts, w.rng_seed, model,
                              None if model == 2 else ws, wn, bs, logits)
        for ln in lanes:
            ln.ctx.sync()
        for k, ln in enumerate(lanes):
            _check_lane(gu, ln, *want[first + k])
    out = logits.cpu().numpy()
    for b in range(nb):
        _check_logits(out[b * B:(b + 1) * B], ref[b])


def test_fused_input_lanes_give_the_same_logits(setup):
    """DCI_OPT_FUSED_INPUT on every lane: cached neighbour rows are read in place; logits of all sixteen batches
    against the oracle, blocks bit for bit, statistics as with the two-call route."""
    dci, gu, w, g, cache, lanes, want, tiny = (setup[k] for k in ("dci", "gu", "w", "g", "cache", "lanes", "want", "tiny"))
    ws, wn, bs = setup["weights"]
    nb = len(want)
    logits = torch.full((w.num_seeds, w.classes), float("nan"), dtype=torch.float32, device="cuda")
    stats = gu.new_stats()
    torch.cuda.synchronize()
    for ln in lanes:
        ln.ctx.set_option(dci.DCI_OPT_FUSED_INPUT, 1)
    try:
        dci.dci_infer_batches(lanes, g, cache, setup["seeds"], B, 0, nb, w.fanouts, w.rng_seed, 0, ws, wn, bs, logits, stats)
        for ln in lanes:
            ln.ctx.sync()
    finally:
        for ln in lanes:
            ln.ctx.set_option(dci.DCI_OPT_FUSED_INPUT, 0)
    out = logits.cpu().numpy()
    for b, (blk, x) in enumerate(want):
        _check_logits(out[b * B:(b + 1) * B], oracle.sage_forward(blk, x, tiny["w_self"], tiny["w_neigh"], tiny["bias"]))
    for k, ln in enumerate(lanes):
        gu.assert_blocks_equal(gu.blocks_to_host(ln.ctx, ln.blocks), want[nb - N_LANES + k][0])
    st = {k: int(v) for k, v in zip(dci.STAT.keys(), stats.cpu().numpy())}
    hits = sum(int((setup["feat_remap"][blk.nodes] >= 0).sum()) for blk, _ in want)
    assert (st["feat_hits"], st["feat_hits"] + st["feat_misses"]) == (hits, sum(len(blk.nodes) for blk, _ in want))


def test_ragged_last_batch_and_ranges(setup):
    """A seed list that ends inside a batch, a range that runs past the last batch, an empty range, one lane."""
    dci, gu, w, g, cache, lanes, tiny = (setup[k] for k in ("dci", "gu", "w", "g", "cache", "lanes", "tiny"))
    ws, wn, bs = setup["weights"]
    n = 5 * B + 37
    seeds = setup["seeds"][:n]
    logits = torch.full((n, w.classes), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    dci.dci_infer_batches(lanes[:3], g, cache, seeds, B, 2, 0, w.fanouts, w.rng_seed, 0, ws, wn, bs, logits)   # nothing
    dci.dci_infer_batches(lanes[:3], g, cache, seeds, B, 2, 100, w.fanouts, w.rng_seed, 0, ws, wn, bs, logits)  # 2..5
    dci.dci_infer_batches(lanes[3:], g, cache, seeds, B, 0, 2, w.fanouts, w.rng_seed, 0, ws, wn, bs, logits)    # 0, 1
    for ln in lanes:
        ln.ctx.sync()
    out = logits.cpu().numpy()
    assert not np.isnan(out).any()
    for b in range(6):
        s = tiny["seeds"][b * B:min(n, (b + 1) * B)]
        blk = oracle.sample_khop(tiny["indptr"], tiny["indices"], s, b, w.fanouts, w.rng_seed)
        ref = oracle.sage_forward(blk, oracle.gather(tiny["feat"], blk.nodes), tiny["w_self"], tiny["w_neigh"], tiny["bias"])
        _check_logits(out[b * B:b * B + len(s)], ref)
    # of the three lanes, lane 0 ran batches 2 and 5: it holds the ragged last batch (37 seeds)
    last = oracle.sample_khop(tiny["indptr"], tiny["indices"], tiny["seeds"][5 * B:n], 5, w.fanouts, w.rng_seed)
    assert last.n_nodes[0] == 37
    _check_lane(gu, lanes[0], last, oracle.gather(tiny["feat"], last.nodes))


def test_lanes_must_not_share(setup):
    dci, w, g, cache, lanes = (setup[k] for k in ("dci", "w", "g", "cache", "lanes"))
    ws, wn, bs = setup["weights"]
    logits = torch.empty(w.num_seeds, w.classes, dtype=torch.float32, device="cuda")
    with pytest.raises(dci.DciError) as e:
        dci.dci_infer_batches([lanes[0], lanes[0]], g, cache, setup["seeds"], B, 0, 2, w.fanouts, w.rng_seed, 0, ws, wn, bs,
                              logits)
    assert e.value.code == -1 and "share" in str(e.value)
