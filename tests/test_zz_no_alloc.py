"""The sampler entry point that allocates nothing (dci_sample_khop_static: temporaries in the
library's static device array) against dci_sample_khop, through the C boundary.

Two calls in a row on one context, the second with a smaller batch, so that the second call runs over
whatever the first one left in the shared array; every output array and the statistics must be
identical, bit for bit, to those of the workspace-based entry point and to the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu


def _run(dci, gu, entry, ctx, g, cache, seeds, b, w, blk):
    stats = gu.new_stats()
    entry(ctx, g, cache, gu.dev(seeds), b, w.fanouts, w.rng_seed, blk, stats)
    got = gu.blocks_to_host(ctx, blk)
    return got, gu.stats_dict(ctx, stats)


@pytest.mark.parametrize("with_cache", [False, True])
def test_static_scratch_sampler_matches_the_workspace_sampler(tiny, with_cache):
    import paper_2503_01281_amd as dci
    from tests import gpu_util as gu
    w = tiny["w"]
    ctx = dci.Context(0)
    g = gu.make_graph(tiny["indptr"], tiny["indices"], tiny["feat"])
    cache = None
    if with_cache:
        fc = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
        ac = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
        dci.dci_presample_count(ctx, g, None, gu.dev(tiny["seeds"]), w.batch_size, 0, w.n_presample,
                                w.presample_first_batch, w.fanouts, w.rng_seed, fc, ac)
        cache = dci.dci_fill_caches(ctx, g, fc, ac, w.budget_bytes, 3, 7, 0)
    blk_a = dci.Blocks(ctx, w.num_nodes, w.batch_size, w.fanouts)
    blk_b = dci.Blocks(ctx, w.num_nodes, w.batch_size, w.fanouts)
    # a second context on the same GPU must see the same array
    ctx2 = dci.Context(0)
    # first call: a full batch; second call: a smaller one (ragged: 77 seeds), then a one-seed batch
    for call, (b, lo, n, c) in enumerate([(0, 0, w.batch_size, ctx), (3, 3 * w.batch_size, 77, ctx),
                                          (5, 5 * w.batch_size, 1, ctx2)]):
        seeds = tiny["seeds"][lo:lo + n]
        got_s, st_s = _run(dci, gu, dci.dci_sample_khop_static, c, g, cache, seeds, b, w, blk_a)
        got_w, st_w = _run(dci, gu, dci.dci_sample_khop, c, g, cache, seeds, b, w, blk_b)
        want = oracle.sample_khop(tiny["indptr"], tiny["indices"], seeds, b, w.fanouts, w.rng_seed)
        gu.assert_blocks_equal(got_s, want)
        gu.assert_blocks_equal(got_w, want)
        assert got_s["n_nodes"] == got_w["n_nodes"] and got_s["n_edges"] == got_w["n_edges"], call
        assert np.array_equal(got_s["nodes"], got_w["nodes"])
        for h in range(w.n_hops):
            assert np.array_equal(got_s["blk_indptr"][h], got_w["blk_indptr"][h])
            assert np.array_equal(got_s["blk_src"][h], got_w["blk_src"][h])
        assert st_s == st_w, (call, st_s, st_w)


def test_static_scratch_sampler_medium_sized_batch_and_size_limit():
    """A batch with the bounds of the Medium workload (close to the array's limit) on a small graph, then a
    smaller one; and a batch whose bounds exceed the array is refused with DCI_ERR_CAPACITY, nothing launched."""
    import paper_2503_01281_amd as dci
    from tests import gpu_util as gu
    n, e = 200_000, 3_000_000
    indptr, indices = synth.rmat_csr(n, e, (0.57, 0.19, 0.19), 21)
    seeds = synth.seeds(n, 6000, 22)
    fan = (5, 10, 15)
    ctx = dci.Context(0)
    g = gu.make_graph(indptr, indices, None, on_device=True)
    blk_a = dci.Blocks(ctx, n, 1024, fan)
    blk_b = dci.Blocks(ctx, n, 1024, fan)
    for b, lo, k in [(0, 0, 1024), (1, 1024, 300)]:
        s = seeds[lo:lo + k]
        dci.dci_sample_khop_static(ctx, g, None, gu.dev(s), b, fan, 9, blk_a)
        got_s = gu.blocks_to_host(ctx, blk_a)
        dci.dci_sample_khop(ctx, g, None, gu.dev(s), b, fan, 9, blk_b)
        got_w = gu.blocks_to_host(ctx, blk_b)
        want = oracle.sample_khop(indptr, indices, s, b, fan, 9)
        gu.assert_blocks_equal(got_s, want)
        gu.assert_blocks_equal(got_w, want)
    big = dci.Blocks(ctx, n, 4096, fan)
    with pytest.raises(dci.DciError) as err:
        dci.dci_sample_khop_static(ctx, g, None, gu.dev(seeds[:4096]), 0, fan, 9, big)
    assert err.value.code == -2 and "static scratch" in str(err.value)
    # the refused call left the context usable
    dci.dci_sample_khop_static(ctx, g, None, gu.dev(seeds[:50]), 2, fan, 9, blk_a)
    gu.assert_blocks_equal(gu.blocks_to_host(ctx, blk_a), oracle.sample_khop(indptr, indices, seeds[:50], 2, fan, 9))
