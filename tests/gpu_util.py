"""Helpers shared by the GPU parity tests: move synthetic inputs to the GPU machine's memory and
bring results back as numpy arrays."""
import numpy as np
import torch

import paper_2503_01281_amd as dci


def pinned(a: np.ndarray) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a))
    return t.pin_memory()


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def make_graph(indptr, indices, feat, on_device=False) -> dci.Graph:
    mv = dev if on_device else pinned
    return dci.Graph(mv(indptr), mv(indices), None if feat is None else mv(feat))


def upload_cache(adj_remap, c_indptr, c_indices, feat_remap, feat_cache, partial_node=-1, partial_deg=0) -> dci.Cache:
    if len(c_indices) == 0:
        c_indices = np.zeros(1, dtype=np.int64)[:0]
    return dci.Cache.from_arrays(dev(adj_remap.astype(np.int32)), dev(c_indptr.astype(np.int64)),
                                 torch.from_numpy(np.ascontiguousarray(c_indices, dtype=np.int64)).cuda(),
                                 dev(feat_remap.astype(np.int32)),
                                 torch.from_numpy(np.ascontiguousarray(feat_cache, dtype=np.float32)).cuda(),
                                 partial_node, partial_deg)


def blocks_to_host(ctx, blk: dci.Blocks):
    ctx.sync()
    nn, ne = blk.n_nodes(), blk.n_edges()
    L = blk.n_hops
    return dict(n_nodes=nn, n_edges=ne, nodes=blk.nodes[:nn[L]].cpu().numpy(),
                blk_indptr=[blk.blk_indptr[h][:nn[h] + 1].cpu().numpy() for h in range(L)],
                blk_src=[blk.blk_src[h][:ne[h]].cpu().numpy() for h in range(L)])


def assert_blocks_equal(got, want):
    """got: dict from blocks_to_host; want: oracle.Blocks.  Bit-exact."""
    assert got["n_nodes"] == [int(x) for x in want.n_nodes]
    assert got["n_edges"] == [int(x) for x in want.n_edges]
    assert np.array_equal(got["nodes"], want.nodes)
    for h in range(len(want.blk_indptr)):
        assert np.array_equal(got["blk_indptr"][h], want.blk_indptr[h]), f"blk_indptr hop {h}"
        assert np.array_equal(got["blk_src"][h], want.blk_src[h]), f"blk_src hop {h}"


def new_stats():
    return torch.zeros(dci.STATS_WORDS, dtype=torch.int64, device="cuda")


def stats_dict(ctx, stats):
    ctx.sync()
    s = stats.cpu().numpy()
    return {k: int(s[i]) for k, i in dci.STAT.items()}
