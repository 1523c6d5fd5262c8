"""A whole step (sample -> gather -> forward) recorded into a HIP graph and replayed.

The library launches kernels only on this path (buffers are cleared by fill kernels, sizes stay on the device,
nothing waits), so the step can be captured once and replayed with new seeds in the same device buffer.  Every
replay is checked against the eager result, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("variant", ["workspace", "static_scratch_and_rows_in_place"])
def test_step_replays_from_a_hip_graph(tiny, variant):
    import paper_2503_01281_amd as dci
    from tests import gpu_util as gu
    w = tiny["w"]
    side = torch.cuda.Stream()
    ctx = dci.Context(0, stream=side)
    g = gu.make_graph(tiny["indptr"], tiny["indices"], tiny["feat"])
    with torch.cuda.stream(side):
        fc = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
        ac = torch.zeros(w.num_nodes, dtype=torch.int32, device="cuda")
        all_seeds = gu.dev(tiny["seeds"])
        dci.dci_presample_count(ctx, g, None, all_seeds, w.batch_size, 0, w.n_presample, w.presample_first_batch, w.fanouts,
                                w.rng_seed, fc, ac)
        cache = dci.dci_fill_caches(ctx, g, fc, ac, w.budget_bytes, 3, 7, 0)
        blk = dci.Blocks(ctx, w.num_nodes, w.batch_size, w.fanouts)
        x = torch.empty(blk.cap_nodes[-1], w.feat_dim, dtype=torch.float32, device="cuda")
        logits = torch.empty(w.batch_size, w.classes, dtype=torch.float32, device="cuda")
        seeds = torch.empty(w.batch_size, dtype=torch.int64, device="cuda")
        ws, wn, bs = ([gu.dev(a) for a in tiny[k]] for k in ("w_self", "w_neigh", "bias"))
        batch_index = 5

        def step():
            if variant == "workspace":
                dci.dci_sample_khop(ctx, g, cache, seeds, batch_index, w.fanouts, w.rng_seed, blk)
                dci.dci_gather_features(ctx, g, cache, blk.nodes, blk.cap_nodes[-1], x, n_dev=blk.n_input_dev())
                dci.dci_sage_forward(ctx, blk, x, ws, wn, bs, logits)
            else:
                # the sampler that allocates nothing (temporaries in the library's static device array), then the
                # gather + forward that reads cached rows in place: x then holds only missed rows and those of F_{L-1}
                dci.dci_sample_khop_static(ctx, g, cache, seeds, batch_index, w.fanouts, w.rng_seed, blk)
                dci.dci_gather_forward(ctx, g, cache, blk, x, dci.DCI_MODEL_SAGE_MEAN, ws, wn, bs, logits)

        def snapshot():
            ctx.sync()
            got = gu.blocks_to_host(ctx, blk)
            return got, x[:got["n_nodes"][-1]].cpu().numpy().copy(), logits.cpu().numpy().copy()

        def scribble():
            blk.nodes.fill_(-1); blk.counts.fill_(-1); x.fill_(0.5); logits.fill_(float("nan"))
            for t in blk.blk_src:
                t.fill_(-1)

        seeds.copy_(all_seeds[:w.batch_size])
        step()                                   # eager once: sizes the workspace before the capture
        ctx.sync()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        for r, lo in enumerate([0, 256, 512, 0, 768]):
            seeds_np = tiny["seeds"][lo:lo + w.batch_size]
            seeds.copy_(all_seeds[lo:lo + w.batch_size])
            scribble()
            step()                               # eager reference on the same buffers
            want = snapshot()
            scribble()
            torch.cuda.synchronize()
            graph.replay()
            got = snapshot()
            assert got[0]["n_nodes"] == want[0]["n_nodes"] and got[0]["n_edges"] == want[0]["n_edges"], f"replay {r}"
            assert np.array_equal(got[0]["nodes"], want[0]["nodes"])
            for h in range(w.n_hops):
                assert np.array_equal(got[0]["blk_indptr"][h], want[0]["blk_indptr"][h])
                assert np.array_equal(got[0]["blk_src"][h], want[0]["blk_src"][h])
            assert got[1].tobytes() == want[1].tobytes() and got[2].tobytes() == want[2].tobytes(), f"replay {r}"
            # and the eager result is the oracle's
            ob = oracle.sample_khop(tiny["indptr"], tiny["indices"], seeds_np, batch_index, w.fanouts, w.rng_seed)
            gu.assert_blocks_equal(want[0], ob)
            ol = oracle.sage_forward(ob, oracle.gather(tiny["feat"], ob.nodes), tiny["w_self"], tiny["w_neigh"], tiny["bias"])
            assert float(np.abs(got[2] - ol).max()) <= 1e-4 * max(1.0, float(np.abs(ol).max()))
