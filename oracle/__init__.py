"""ctypes front end of the CPU oracle (``dci_oracle.cpp``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The product path never imports this package, and this
package imports nothing from the product path.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dci_oracle.cpp")
_LIB = os.environ.get("DCI_ORACLE_LIB") or os.path.join(_HERE, "libdci_oracle.so")  # override: mutation checks of the pins
_lib = None

c = ctypes
_P = c.c_void_p


SANITIZE_FLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-pthread", "-o", _LIB, _SRC], check=True)
    return _LIB


def build_sanitized() -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (host code only); load it by
    pointing DCI_ORACLE_LIB at the result in a process that has the sanitizer runtime preloaded."""
    out = os.path.join(_HERE, "libdci_oracle_asan.so")
    subprocess.run(["g++", "-std=c++17", "-fPIC", "-shared", "-pthread"] + SANITIZE_FLAGS + ["-o", out, _SRC], check=True)
    return out


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        lib = c.CDLL(_LIB)
        lib.oracle_philox4x32_10.argtypes = [_P, _P, _P]
        lib.oracle_philox4x32_10.restype = None
        lib.oracle_uniform_below.argtypes = [c.c_uint64, c.c_int64, c.c_uint64, c.c_int32, c.c_int32, c.c_uint64]
        lib.oracle_uniform_below.restype = c.c_uint64
        lib.oracle_sample_positions.argtypes = [c.c_uint64, c.c_uint64, c.c_int32, c.c_int64, c.c_int64,
                                                c.c_int32, _P]
        lib.oracle_sample_positions.restype = c.c_int32
        lib.oracle_sample_khop.argtypes = [_P, _P, _P, c.c_int64, c.c_uint64, _P, c.c_int32, c.c_uint64,
                                           _P, c.c_int64, _P, _P, _P, _P, _P, _P, _P]
        lib.oracle_sample_khop.restype = c.c_int32
        lib.oracle_presample_count.argtypes = [_P, _P, _P, c.c_int64, c.c_int32, c.c_int64, c.c_int64,
                                               c.c_uint64, _P, c.c_int32, c.c_uint64, _P, _P, _P, _P]
        lib.oracle_presample_count.restype = c.c_int32
        lib.oracle_split.argtypes = [c.c_uint64, c.c_uint64, c.c_uint64, c.c_int64, c.c_int64, c.c_int32, c.c_int32, _P, _P]
        lib.oracle_split.restype = None
        lib.oracle_fill_feat.argtypes = [c.c_int64, c.c_int32, _P, _P, c.c_uint64, c.c_int32, _P, _P]
        lib.oracle_fill_feat.restype = c.c_int64
        lib.oracle_fill_adj.argtypes = [c.c_int64, _P, _P, _P, c.c_uint64, _P, _P, c.c_int64, _P, c.c_int64,
                                        _P, _P]
        lib.oracle_fill_adj.restype = c.c_int32
        lib.oracle_gather.argtypes = [_P, c.c_int32, _P, c.c_int64, _P]
        lib.oracle_gather.restype = None
        lib.oracle_gather_cached.argtypes = [_P, c.c_int32, _P, _P, _P, c.c_int64, _P, _P]
        lib.oracle_gather_cached.restype = None
        lib.oracle_sample_hop_cached.argtypes = [_P, _P, _P, _P, _P, c.c_int64, c.c_int64, _P, c.c_int64,
                                                 c.c_uint64, c.c_int32, c.c_int32, c.c_uint64, _P, _P, _P]
        lib.oracle_fill_adj_element.argtypes = [c.c_int64, _P, _P, _P, c.c_uint64, _P, _P, c.c_int64, _P,
                                                c.c_int64, _P, _P, _P, _P]
        lib.oracle_fill_adj_element.restype = c.c_int32
        lib.oracle_sample_hop_cached.restype = c.c_int32
        lib.oracle_sage_forward.argtypes = [c.c_int32, _P, _P, _P, _P, _P, _P, _P, _P, _P]
        lib.oracle_sage_forward.restype = None
        lib.oracle_gnn_forward.argtypes = [c.c_int32, c.c_int32, _P, _P, _P, _P, _P, _P, _P, _P, _P]
        lib.oracle_gnn_forward.restype = None
        lib.oracle_run_batches.argtypes = [_P, _P, _P, c.c_int32, _P, c.c_int64, c.c_int32, c.c_int64, c.c_int64, _P,
                                           c.c_int32, c.c_uint64, c.c_int32, _P, _P, _P, _P, c.c_int32, _P]
        lib.oracle_run_batches.restype = c.c_int32
        _lib = lib
    return _lib


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int64)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr_array(arrs: Sequence[Optional[np.ndarray]]):
    pa = (c.c_void_p * len(arrs))()
    for i, a in enumerate(arrs):
        pa[i] = None if a is None else a.ctypes.data
    return pa


def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> List[int]:
    lib = _load()
    cc = np.array(ctr, dtype=np.uint32)
    kk = np.array(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib.oracle_philox4x32_10(cc.ctypes.data, kk.ctypes.data, out.ctypes.data)
    return [int(x) for x in out]


def uniform_below(rng_seed: int, node: int, batch_index: int, hop: int, slot: int, m: int) -> int:
    return int(_load().oracle_uniform_below(rng_seed, node, batch_index, hop, slot, m))


def sample_positions(rng_seed: int, batch_index: int, hop: int, node: int, deg: int, fanout: int) -> np.ndarray:
    pos = np.zeros(max(fanout, deg if deg <= fanout else fanout, 1), dtype=np.int64)
    n = _load().oracle_sample_positions(rng_seed, batch_index, hop, node, deg, fanout, pos.ctypes.data)
    return pos[:n].copy()


@dataclass
class Blocks:
    """One sampled mini-batch (host arrays)."""
    n_nodes: np.ndarray           # [L+1]
    n_edges: np.ndarray           # [L]
    nodes: np.ndarray             # F_L, int64
    blk_indptr: List[np.ndarray]  # per hop, int64 [n_nodes[h]+1]
    blk_src: List[np.ndarray]     # per hop, int32 [n_edges[h]] local ids into F_{h+1}
    src_global: List[np.ndarray]  # per hop, int64 [n_edges[h]]
    src_pos: List[np.ndarray]     # per hop, int64 [n_edges[h]] position in the node's list


def sample_khop(indptr, indices, seeds, batch_index: int, fanouts: Sequence[int], rng_seed: int,
                num_nodes: Optional[int] = None) -> Blocks:
    lib = _load()
    indptr, indices, seeds = _i64(indptr), _i64(indices), _i64(seeds)
    N = len(indptr) - 1 if num_nodes is None else num_nodes
    L = len(fanouts)
    fo = _i32(fanouts)
    caps_n = [len(seeds)]
    for f in fanouts:
        caps_n.append(caps_n[-1] * (1 + f))
    cap_e = [caps_n[h] * fanouts[h] for h in range(L)]
    nodes = np.empty(max(caps_n[-1], 1), dtype=np.int64)
    n_nodes = np.zeros(L + 1, dtype=np.int64)
    n_edges = np.zeros(L, dtype=np.int64)
    bi = [np.empty(caps_n[h] + 1, dtype=np.int64) for h in range(L)]
    bs = [np.empty(max(cap_e[h], 1), dtype=np.int32) for h in range(L)]
    sg = [np.empty(max(cap_e[h], 1), dtype=np.int64) for h in range(L)]
    sp = [np.empty(max(cap_e[h], 1), dtype=np.int64) for h in range(L)]
    ce = _i64(cap_e)
    rc = lib.oracle_sample_khop(indptr.ctypes.data, indices.ctypes.data, seeds.ctypes.data, len(seeds),
                                batch_index, fo.ctypes.data, L, rng_seed, nodes.ctypes.data, len(nodes),
                                n_nodes.ctypes.data, n_edges.ctypes.data, _ptr_array(bi), _ptr_array(bs),
                                _ptr_array(sg), _ptr_array(sp), ce.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_sample_khop failed: {rc}")
    return Blocks(n_nodes=n_nodes, n_edges=n_edges, nodes=nodes[:n_nodes[L]].copy(),
                  blk_indptr=[bi[h][:n_nodes[h] + 1].copy() for h in range(L)],
                  blk_src=[bs[h][:n_edges[h]].copy() for h in range(L)],
                  src_global=[sg[h][:n_edges[h]].copy() for h in range(L)],
                  src_pos=[sp[h][:n_edges[h]].copy() for h in range(L)])


def presample_count(indptr, indices, seeds, batch_size: int, n_batches: int, fanouts: Sequence[int],
                    rng_seed: int, rng_batch0: int, first_batch: int = 0, with_edge_count: bool = True,
                    feat_count=None, adj_count=None, edge_count=None):
    """Returns (feat_count[N], adj_count[N], edge_count[E] or None, (edges, input_nodes))."""
    lib = _load()
    indptr, indices, seeds = _i64(indptr), _i64(indices), _i64(seeds)
    N, E = len(indptr) - 1, len(indices)
    fo = _i32(fanouts)
    fc = np.zeros(N, dtype=np.uint32) if feat_count is None else feat_count
    ac = np.zeros(N, dtype=np.uint32) if adj_count is None else adj_count
    ec = None
    if with_edge_count:
        ec = np.zeros(max(E, 1), dtype=np.uint32)[:E] if edge_count is None else edge_count
    totals = np.zeros(2, dtype=np.int64)
    rc = lib.oracle_presample_count(indptr.ctypes.data, indices.ctypes.data, seeds.ctypes.data, len(seeds),
                                    batch_size, first_batch, n_batches, rng_batch0, fo.ctypes.data, len(fo),
                                    rng_seed, fc.ctypes.data, ac.ctypes.data,
                                    None if ec is None else ec.ctypes.data, totals.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_presample_count failed: {rc}")
    return fc, ac, ec, (int(totals[0]), int(totals[1]))


def split(C: int, t_sample: int, t_feature: int, N: int, E: int, F: int, spill: bool = True):
    a = c.c_uint64(0)
    f = c.c_uint64(0)
    _load().oracle_split(C, t_sample, t_feature, N, E, F, 1 if spill else 0, c.byref(a), c.byref(f))
    return int(a.value), int(f.value)


def fill_feat(feat_count, feat, C_feat: int, policy: int = 0, feat_dim: Optional[int] = None):
    """Returns (feat_remap[N] int32, feat_cache[k,F] or None, k)."""
    lib = _load()
    fc = np.ascontiguousarray(feat_count, dtype=np.uint32)
    N = len(fc)
    F = feat.shape[1] if feat is not None else int(feat_dim)
    k = min(N, C_feat // (4 * F))
    remap = np.empty(N, dtype=np.int32)
    cache = None
    if feat is not None:
        feat = np.ascontiguousarray(feat, dtype=np.float32)
        cache = np.zeros((max(k, 1), F), dtype=np.float32)[:k]
    got = lib.oracle_fill_feat(N, F, fc.ctypes.data, None if feat is None else feat.ctypes.data, C_feat, policy,
                               remap.ctypes.data, None if cache is None else cache.ctypes.data)
    assert got == k
    return remap, cache, int(k)


def fill_adj(indptr, indices, adj_count, C_adj: int):
    """Returns (adj_remap[N] int32, c_indptr[K+1], c_indices[M])."""
    lib = _load()
    indptr, indices = _i64(indptr), _i64(indices)
    ac = np.ascontiguousarray(adj_count, dtype=np.uint32)
    N = len(indptr) - 1
    remap = np.empty(N, dtype=np.int32)
    K = c.c_int64(0)
    M = c.c_int64(0)
    rc = lib.oracle_fill_adj(N, indptr.ctypes.data, indices.ctypes.data, ac.ctypes.data, C_adj,
                             remap.ctypes.data, None, 0, None, 0, c.byref(K), c.byref(M))
    assert rc == 0
    cp = np.zeros(K.value + 1, dtype=np.int64)
    ci = np.zeros(max(M.value, 1), dtype=np.int64)
    rc = lib.oracle_fill_adj(N, indptr.ctypes.data, indices.ctypes.data, ac.ctypes.data, C_adj,
                             remap.ctypes.data, cp.ctypes.data, K.value, ci.ctypes.data, M.value,
                             c.byref(K), c.byref(M))
    assert rc == 0
    return remap, cp, ci[:M.value]


def gather(feat, ids) -> np.ndarray:
    feat = np.ascontiguousarray(feat, dtype=np.float32)
    ids = _i64(ids)
    out = np.empty((len(ids), feat.shape[1]), dtype=np.float32)
    _load().oracle_gather(feat.ctypes.data, feat.shape[1], ids.ctypes.data, len(ids), out.ctypes.data)
    return out


def gather_cached(feat, feat_remap, feat_cache, ids):
    """Returns (rows, hits, misses)."""
    feat = np.ascontiguousarray(feat, dtype=np.float32)
    feat_cache = np.ascontiguousarray(feat_cache, dtype=np.float32)
    remap = _i32(feat_remap)
    ids = _i64(ids)
    out = np.empty((len(ids), feat.shape[1]), dtype=np.float32)
    counts = np.zeros(2, dtype=np.int64)
    _load().oracle_gather_cached(feat.ctypes.data, feat.shape[1], remap.ctypes.data, feat_cache.ctypes.data,
                                 ids.ctypes.data, len(ids), out.ctypes.data, counts.ctypes.data)
    return out, int(counts[0]), int(counts[1])


def fill_adj_element(indptr, indices, edge_count, C_adj: int):
    """Element-granular fill.  Returns (adj_remap[N] int32, c_indptr[K+1], c_indices[M], indices_reordered[E],
    partial_node, partial_deg); the input `indices` is left untouched."""
    lib = _load()
    indptr = _i64(indptr)
    idx = _i64(indices).copy()
    ec = np.ascontiguousarray(edge_count, dtype=np.uint32)
    N = len(indptr) - 1
    remap = np.empty(N, dtype=np.int32)
    K, M, pn, pd = c.c_int64(0), c.c_int64(0), c.c_int64(0), c.c_int64(0)
    cap_M = int(min(len(idx), C_adj // 8))
    cp = np.zeros(N + 1, dtype=np.int64)
    ci = np.zeros(max(cap_M, 1), dtype=np.int64)
    rc = lib.oracle_fill_adj_element(N, indptr.ctypes.data, idx.ctypes.data, ec.ctypes.data, C_adj,
                                     remap.ctypes.data, cp.ctypes.data, N, ci.ctypes.data, cap_M,
                                     c.byref(K), c.byref(M), c.byref(pn), c.byref(pd))
    assert rc == 0
    cp = cp[:K.value + 1].copy()
    return remap, cp, ci[:M.value], idx, int(pn.value), int(pd.value)


def sample_hop_cached(indptr, indices, adj_remap, c_indptr, c_indices, frontier, batch_index: int, hop: int,
                      fanout: int, rng_seed: int, partial_node: int = -1, partial_deg: int = 0):
    """Returns (row_count[n], src_global[sum], counts[4] = nodes with a slot, without, positions from the cache,
    from the host)."""
    indptr, indices, frontier = _i64(indptr), _i64(indices), _i64(frontier)
    c_indptr, c_indices = _i64(c_indptr), _i64(c_indices)
    remap = _i32(adj_remap)
    n = len(frontier)
    rows = np.zeros(max(n, 1), dtype=np.int64)
    src = np.zeros(max(n * fanout, 1), dtype=np.int64)
    counts = np.zeros(4, dtype=np.int64)
    _load().oracle_sample_hop_cached(indptr.ctypes.data, indices.ctypes.data, remap.ctypes.data,
                                     c_indptr.ctypes.data, c_indices.ctypes.data, partial_node, partial_deg,
                                     frontier.ctypes.data, n, batch_index, hop, fanout, rng_seed, rows.ctypes.data,
                                     src.ctypes.data, counts.ctypes.data)
    rows = rows[:n]
    return rows, src[:int(rows.sum())].copy(), counts


SAGE_MEAN, SAGE_SUM, GCN_AVG = 0, 1, 2


def sage_forward(blocks: Blocks, x_in, w_self, w_neigh, bias) -> np.ndarray:
    """fp64 logits [n_nodes[0], dims[-1]] of the GraphSAGE-mean model."""
    return gnn_forward(SAGE_MEAN, blocks, x_in, w_self, w_neigh, bias)


def gnn_forward(model: int, blocks: Blocks, x_in, w_self, w_neigh, bias) -> np.ndarray:
    """fp64 logits [n_nodes[0], dims[-1]]; model = SAGE_MEAN, SAGE_SUM or GCN_AVG (w_self unused)."""
    lib = _load()
    if w_self is None:
        w_self = w_neigh
    L = len(w_self)
    assert L == len(blocks.blk_indptr)
    x_in = np.ascontiguousarray(x_in, dtype=np.float32)
    dims = _i32([w_self[0].shape[0]] + [w.shape[1] for w in w_self])
    assert x_in.shape == (blocks.n_nodes[L], dims[0])
    ws = [np.ascontiguousarray(w, dtype=np.float32) for w in w_self]
    wn = [np.ascontiguousarray(w, dtype=np.float32) for w in w_neigh]
    bb = [np.ascontiguousarray(b, dtype=np.float32) for b in bias]
    bi = [_i64(a) for a in blocks.blk_indptr]
    bs = [_i32(a) if len(a) else np.zeros(1, dtype=np.int32) for a in blocks.blk_src]
    nn = _i64(blocks.n_nodes)
    out = np.zeros((int(nn[0]), int(dims[L])), dtype=np.float64)
    lib.oracle_gnn_forward(model, L, nn.ctypes.data, _ptr_array(bi), _ptr_array(bs), x_in.ctypes.data,
                           dims.ctypes.data, _ptr_array(ws), _ptr_array(wn), _ptr_array(bb), out.ctypes.data)
    return out


def run_batches(indptr, indices, feat, seeds, batch_size: int, first_batch: int, n_batches: int,
                fanouts: Sequence[int], rng_seed: int, model: int, w_self, w_neigh, bias, n_threads: int = 1) -> dict:
    """Whole batches (sample -> gather -> forward) on ``n_threads`` host threads, batch k of the range on thread
    k mod n_threads; returns wall seconds, per-stage seconds summed over the threads, and totals."""
    lib = _load()
    indptr, indices, seeds = _i64(indptr), _i64(indices), _i64(seeds)
    feat = np.ascontiguousarray(feat, dtype=np.float32)
    if w_self is None:
        w_self = w_neigh
    L = len(w_neigh)
    assert L == len(fanouts)
    dims = _i32([w_neigh[0].shape[0]] + [w.shape[1] for w in w_neigh])
    ws = [np.ascontiguousarray(w, dtype=np.float32) for w in w_self]
    wn = [np.ascontiguousarray(w, dtype=np.float32) for w in w_neigh]
    bb = [np.ascontiguousarray(b, dtype=np.float32) for b in bias]
    out = np.zeros(8, dtype=np.float64)
    rc = lib.oracle_run_batches(indptr.ctypes.data, indices.ctypes.data, feat.ctypes.data, int(feat.shape[1]),
                                seeds.ctypes.data, len(seeds), batch_size, first_batch, n_batches,
                                _i32(fanouts).ctypes.data, L, rng_seed, model, dims.ctypes.data, _ptr_array(ws),
                                _ptr_array(wn), _ptr_array(bb), n_threads, out.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_run_batches: bad arguments")
    return dict(wall_s=float(out[0]), sample_s=float(out[1]), gather_s=float(out[2]), forward_s=float(out[3]),
                edges=int(out[4]), input_rows=int(out[5]), batches=int(out[6]), logit_sum=float(out[7]), threads=n_threads)
