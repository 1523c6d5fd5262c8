"""ctypes binding of libdci.so: argument marshalling only, every step runs in the HIP kernels.

There is no fallback: if the library has not been built (``python -m paper_2503_01281_amd.build``
or ``__graft_entry__.build()``) loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

DCI_MAX_HOPS = 8
STATS_WORDS = 16
STAT = dict(edges_sampled=0, adj_node_hits=1, adj_node_misses=2, adj_edge_hits=3, adj_edge_misses=4,
            feat_hits=5, feat_misses=6, input_nodes=7, t_sample_ns=8, t_feature_ns=9, bytes_hbm=10, bytes_host=11,
            lines_bounds=12, lines_ids=13, rows_copied=14)

KERNEL_CLASSES = ["table_clear", "sample", "relabel", "write_src", "gather", "mean_in", "linear_in", "mean", "linear",
                  "count_nodes"]

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdci.so")
_lib = None


class DciError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libdci error {code}: {message}")
        self.code = code


class _Graph(C.Structure):
    _fields_ = [("num_nodes", C.c_int64), ("num_edges", C.c_int64), ("feat_dim", C.c_int32),
                ("indptr", C.c_void_p), ("indices", C.c_void_p), ("feat", C.c_void_p)]


class _Cache(C.Structure):
    _fields_ = [("adj_nodes", C.c_int64), ("adj_edges", C.c_int64), ("feat_rows", C.c_int64),
                ("adj_bytes", C.c_uint64), ("feat_bytes", C.c_uint64), ("cap_adj_bytes", C.c_uint64),
                ("cap_feat_bytes", C.c_uint64), ("adj_remap", C.c_void_p), ("c_indptr", C.c_void_p),
                ("c_indices", C.c_void_p), ("adj_partial_node", C.c_int64), ("adj_partial_deg", C.c_int64),
                ("feat_remap", C.c_void_p), ("feat_cache", C.c_void_p)]


class _Lane(C.Structure):
    _fields_ = [("ctx", C.c_void_p), ("blocks", C.c_void_p), ("x", C.c_void_p)]


class _Blocks(C.Structure):
    _fields_ = [("n_hops", C.c_int32), ("cap_nodes", C.c_int64), ("cap_rows", C.c_int64 * DCI_MAX_HOPS),
                ("cap_edges", C.c_int64 * DCI_MAX_HOPS), ("nodes", C.c_void_p),
                ("blk_indptr", C.c_void_p * DCI_MAX_HOPS), ("blk_src", C.c_void_p * DCI_MAX_HOPS),
                ("counts", C.c_void_p), ("counts_host", C.c_void_p)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it first (python -m paper_2503_01281_amd.build); "
                          "there is no CPU fallback")
    lib = C.CDLL(_LIB_PATH)
    P, i32, i64, u64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_size_t
    lib.dci_create.argtypes = [C.POINTER(P), i32, P, P, sz]
    lib.dci_set_workspace.argtypes = [P, P, sz]
    lib.dci_destroy.argtypes = [P]
    lib.dci_destroy.restype = None
    lib.dci_sync.argtypes = [P]
    lib.dci_last_error.argtypes = [P]
    lib.dci_last_error.restype = C.c_char_p
    lib.dci_blocks_bounds.argtypes = [i64, i64, P, i32, P, P]
    lib.dci_last_required.argtypes = [P, P, P, P]
    lib.dci_last_required.restype = i32
    lib.dci_sample_workspace_bytes.argtypes = [i64, i64, P, i32]
    lib.dci_sample_workspace_bytes.restype = sz
    lib.dci_fill_workspace_bytes.argtypes = [i64]
    lib.dci_fill_workspace_bytes.restype = sz
    lib.dci_fill_elements_workspace_bytes.argtypes = [i64, i64]
    lib.dci_fill_elements_workspace_bytes.restype = sz
    lib.dci_sage_workspace_bytes.argtypes = [P, i32, P]
    lib.dci_sage_workspace_bytes.restype = sz
    lib.dci_presample_count.argtypes = [P, P, P, P, i64, i32, i64, i64, u64, P, i32, u64, P, P, P, P, P]
    lib.dci_fill_caches.argtypes = [P, P, P, P, P, u64, u64, u64, i32, P, P, P, P, P]
    lib.dci_sample_khop.argtypes = [P, P, P, P, i64, u64, P, i32, u64, P, P]
    lib.dci_sample_khop_static.argtypes = [P, P, P, P, i64, u64, P, i32, u64, P, P]
    lib.dci_sample_khop_static.restype = i32
    lib.dci_sample_khop_scratch_bytes.argtypes = [i64, i64, P, i32]
    lib.dci_sample_khop_scratch_bytes.restype = sz
    lib.dci_gather_features.argtypes = [P, P, P, P, i64, P, P, P]
    lib.dci_sage_forward.argtypes = [P, P, P, i32, P, P, P, P, P]
    lib.dci_gnn_forward.argtypes = [P, P, P, i32, P, i32, P, P, P, P]
    lib.dci_gather_forward.argtypes = [P, P, P, P, P, i32, P, i32, P, P, P, P, P]
    lib.dci_gather_forward.restype = i32
    lib.dci_gather_forward_workspace_bytes.argtypes = [i64, P, i32, P]
    lib.dci_gather_forward_workspace_bytes.restype = sz
    lib.dci_infer_batches.argtypes = [P, i32, P, P, P, i64, i32, i64, i64, P, i32, u64, i32, P, P, P, P, P, P]
    lib.dci_infer_batches.restype = i32
    lib.dci_probe_read.argtypes = [P, P, u64, i32, i32, i64, i32, u64, P, P]
    lib.dci_probe_read.restype = i32
    lib.dci_set_option.argtypes = [P, i32, i64]
    lib.dci_timing_enable.argtypes = [P, C.c_uint32]
    lib.dci_timing_read.argtypes = [P, P, P]
    for name in ("dci_set_option", "dci_timing_enable", "dci_timing_read", "dci_create", "dci_set_workspace", "dci_sync", "dci_blocks_bounds", "dci_presample_count",
                 "dci_fill_caches", "dci_sample_khop", "dci_gather_features", "dci_sage_forward",
                 "dci_gnn_forward"):
        getattr(lib, name).restype = i32
    _lib = lib
    return lib


_hip = None


def _hip_runtime():
    """The HIP runtime this process already uses (PyTorch loads it), for pinned host allocations."""
    global _hip
    if _hip is None:
        torch.cuda.init()
        h = C.CDLL("libamdhip64.so.7")
        h.hipHostMalloc.argtypes = [C.POINTER(C.c_void_p), C.c_size_t, C.c_uint]
        h.hipHostMalloc.restype = C.c_int
        h.hipHostFree.argtypes = [C.c_void_p]
        h.hipHostFree.restype = C.c_int
        h.hipGetLastError.restype = C.c_int
        _hip = h
    return _hip


class _PinnedOwner:
    def __init__(self, ptr: int):
        self.ptr = ptr

    def __del__(self):
        try:
            if self.ptr and _hip is not None:
                _hip.hipHostFree(C.c_void_p(self.ptr))
        except Exception:
            pass
        self.ptr = 0


def pinned_empty(numel: int, dtype: torch.dtype) -> torch.Tensor:
    """Uninitialised pinned (page-locked, device-mapped) host tensor of exactly ``numel`` elements.

    ``torch.empty(..., pin_memory=True)`` rounds an allocation up to the next power of two, which for the
    tens-of-gigabytes arrays of the host-resident workloads asks for more page-locked memory than a machine
    grants; this takes the exact size from hipHostMalloc.  The memory is freed when the last tensor that
    shares it is gone.  Raises MemoryError if the runtime refuses."""
    nbytes = int(numel) * torch.empty(0, dtype=dtype).element_size()
    if nbytes == 0:
        return torch.empty(0, dtype=dtype)
    h = _hip_runtime()
    p = C.c_void_p()
    rc = h.hipHostMalloc(C.byref(p), nbytes, 0)
    if rc != 0 or not p.value:
        h.hipGetLastError()
        raise MemoryError(f"hipHostMalloc of {nbytes} bytes failed with HIP error {rc}")
    arr = (C.c_char * nbytes).from_address(p.value)
    arr._owner = _PinnedOwner(p.value)
    return torch.frombuffer(arr, dtype=dtype)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _i32_array(values: Sequence[int]):
    return (C.c_int32 * len(values))(*[int(v) for v in values])


def blocks_bounds(num_nodes: int, n_seeds: int, fanouts: Sequence[int]):
    lib = load_library()
    L = len(fanouts)
    cn = (C.c_int64 * (DCI_MAX_HOPS + 1))()
    ce = (C.c_int64 * DCI_MAX_HOPS)()
    rc = lib.dci_blocks_bounds(num_nodes, n_seeds, _i32_array(fanouts), L, cn, ce)
    if rc != 0:
        raise DciError(rc, "dci_blocks_bounds: invalid fan-outs or sizes")
    return [int(cn[h]) for h in range(L + 1)], [int(ce[h]) for h in range(L)]


class Context:
    """A libdci context on a PyTorch stream of ``device`` (default: the current one) with a growable
    workspace.  Calls that involve PyTorch allocations should be made with that stream current."""

    def __init__(self, device: int = 0, workspace_bytes: int = 0, stream: Optional["torch.cuda.Stream"] = None):
        self.lib = load_library()
        self.device = torch.device("cuda", device)
        torch.cuda.set_device(self.device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        self._h = C.c_void_p()
        rc = self.lib.dci_create(C.byref(self._h), device, C.c_void_p(self.stream.cuda_stream), None, 0)
        if rc != 0:
            raise DciError(rc, "dci_create failed")
        self._ws = None
        if workspace_bytes:
            self.ensure_workspace(workspace_bytes)

    @property
    def handle(self):
        return self._h

    def check(self, rc: int):
        if rc != 0:
            raise DciError(rc, self.lib.dci_last_error(self._h).decode())

    def ensure_workspace(self, nbytes: int):
        if self._ws is None or self._ws.numel() < nbytes:
            self.sync()
            self._ws = torch.empty(int(nbytes) + 256, dtype=torch.uint8, device=self.device)
            base = self._ws.data_ptr()
            off = (-base) % 256
            self.check(self.lib.dci_set_workspace(self._h, base + off, self._ws.numel() - 256))

    def sync(self):
        self.check(self.lib.dci_sync(self._h))

    def last_required(self):
        """(cap_nodes[9], cap_edges[8], temporaries in bytes) that the last sampling call on this context needed."""
        cn = (C.c_int64 * (DCI_MAX_HOPS + 1))()
        ce = (C.c_int64 * DCI_MAX_HOPS)()
        ws = C.c_size_t(0)
        self.check(self.lib.dci_last_required(self._h, cn, ce, C.byref(ws)))
        return [int(v) for v in cn], [int(v) for v in ce], int(ws.value)

    def set_option(self, option: int, value: int):
        self.check(self.lib.dci_set_option(self._h, int(option), int(value)))

    def timing_enable(self, classes):
        """classes: iterable of kernel-class names from KERNEL_CLASSES (empty = off)."""
        mask = 0
        for name in classes:
            mask |= 1 << KERNEL_CLASSES.index(name)
        self.check(self.lib.dci_timing_enable(self._h, mask))

    def timing_read(self):
        """{class: (total_ms, launches)} since the last read; waits for the stream."""
        ms = (C.c_double * len(KERNEL_CLASSES))()
        n = (C.c_int64 * len(KERNEL_CLASSES))()
        self.check(self.lib.dci_timing_read(self._h, ms, n))
        return {k: (float(ms[i]), int(n[i])) for i, k in enumerate(KERNEL_CLASSES)}

    def close(self):
        if self._h:
            self.lib.dci_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Graph:
    """Borrowed graph arrays: int64 ``indptr`` [N+1], int64 ``indices`` [E], fp32 ``feat`` [N,F].
    Tensors may be pinned host memory (zero-copy) or device memory."""

    def __init__(self, indptr: torch.Tensor, indices: torch.Tensor, feat: Optional[torch.Tensor], feat_dim: Optional[int] = None):
        assert indptr.dtype == torch.int64 and indices.dtype == torch.int64
        for t in (indptr, indices, feat):
            assert t is None or t.is_contiguous()
            assert t is None or t.numel() == 0 or t.is_cuda or t.is_pinned(), "graph arrays must be pinned host or device memory"
        self.indptr, self.indices, self.feat = indptr, indices, feat
        self.num_nodes = indptr.numel() - 1
        self.num_edges = indices.numel()
        self.feat_dim = int(feat.shape[1]) if feat is not None else int(feat_dim or 1)
        self.c = _Graph(self.num_nodes, self.num_edges, self.feat_dim, _ptr(indptr), _ptr(indices), _ptr(feat))


class Cache:
    """Result of dci_fill_caches: the descriptor plus the tensors that back it."""

    def __init__(self, c: _Cache, keep):
        self.c = c
        self._keep = keep

    adj_nodes = property(lambda s: s.c.adj_nodes)
    adj_edges = property(lambda s: s.c.adj_edges)
    feat_rows = property(lambda s: s.c.feat_rows)
    adj_bytes = property(lambda s: s.c.adj_bytes)
    feat_bytes = property(lambda s: s.c.feat_bytes)
    cap_adj_bytes = property(lambda s: s.c.cap_adj_bytes)
    cap_feat_bytes = property(lambda s: s.c.cap_feat_bytes)
    adj_partial_node = property(lambda s: s.c.adj_partial_node)
    adj_partial_deg = property(lambda s: s.c.adj_partial_deg)

    @staticmethod
    def from_arrays(adj_remap, c_indptr, c_indices, feat_remap, feat_cache, partial_node: int = -1,
                    partial_deg: int = 0) -> "Cache":
        """Wraps cache arrays built elsewhere (device tensors)."""
        K, M, k = c_indptr.numel() - 1, c_indices.numel(), feat_cache.shape[0]
        F = feat_cache.shape[1]
        c = _Cache(K, M, k, 8 * (K + 1) + 8 * M, 4 * F * k, 0, 0, _ptr(adj_remap), _ptr(c_indptr),
                   _ptr(c_indices), partial_node, partial_deg, _ptr(feat_remap), _ptr(feat_cache))
        return Cache(c, (adj_remap, c_indptr, c_indices, feat_remap, feat_cache))


class Blocks:
    """Device buffers of one mini-batch, allocated at the bounds for (n_seeds, fanouts)."""

    def __init__(self, ctx: Context, num_nodes: int, n_seeds: int, fanouts: Sequence[int]):
        self.fanouts = [int(f) for f in fanouts]
        L = len(fanouts)
        self.n_hops = L
        self.cap_nodes, self.cap_edges = blocks_bounds(num_nodes, n_seeds, fanouts)
        dev = ctx.device
        self.nodes = torch.empty(max(self.cap_nodes[L], 1), dtype=torch.int64, device=dev)
        self.blk_indptr = [torch.empty(self.cap_nodes[h] + 1, dtype=torch.int64, device=dev) for h in range(L)]
        self.blk_src = [torch.empty(max(self.cap_edges[h], 1), dtype=torch.int32, device=dev) for h in range(L)]
        self.counts = torch.zeros(2 * DCI_MAX_HOPS + 1, dtype=torch.int64, device=dev)
        self.counts_host = torch.zeros(2 * DCI_MAX_HOPS + 1, dtype=torch.int64).pin_memory()
        c = _Blocks()
        c.n_hops = L
        c.cap_nodes = self.cap_nodes[L]
        for h in range(L):
            c.cap_rows[h] = self.cap_nodes[h]
            c.cap_edges[h] = self.cap_edges[h]
            c.blk_indptr[h] = self.blk_indptr[h].data_ptr()
            c.blk_src[h] = self.blk_src[h].data_ptr()
        c.nodes = self.nodes.data_ptr()
        c.counts = self.counts.data_ptr()
        c.counts_host = self.counts_host.data_ptr()
        self.c = c

    def n_nodes(self) -> List[int]:
        """Valid after a sync."""
        return [int(self.counts_host[h]) for h in range(self.n_hops + 1)]

    def n_edges(self) -> List[int]:
        return [int(self.counts_host[DCI_MAX_HOPS + 1 + h]) for h in range(self.n_hops)]

    def n_input_dev(self) -> int:
        """Device address of n_nodes[L]."""
        return self.counts.data_ptr() + 8 * self.n_hops


def dci_presample_count(ctx: Context, graph: Graph, cache: Optional[Cache], seeds: torch.Tensor, batch_size: int,
                        first_batch: int, n_batches: int, rng_batch0: int, fanouts: Sequence[int], rng_seed: int,
                        feat_count: torch.Tensor, adj_count: torch.Tensor, edge_count: Optional[torch.Tensor] = None,
                        feat_scratch: Optional[torch.Tensor] = None, stats: Optional[torch.Tensor] = None):
    assert seeds.is_cuda and seeds.dtype == torch.int64
    assert feat_count.dtype == torch.int32 or feat_count.dtype == torch.uint32
    ctx.ensure_workspace(ctx.lib.dci_sample_workspace_bytes(graph.num_nodes, batch_size, _i32_array(fanouts), len(fanouts)))
    ctx.check(ctx.lib.dci_presample_count(
        ctx.handle, C.byref(graph.c), None if cache is None else C.byref(cache.c), _ptr(seeds), seeds.numel(),
        batch_size, first_batch, n_batches, rng_batch0, _i32_array(fanouts), len(fanouts), rng_seed,
        _ptr(feat_count), _ptr(adj_count), _ptr(edge_count), _ptr(feat_scratch), _ptr(stats)))


def dci_fill_caches(ctx: Context, graph: Graph, feat_count: torch.Tensor, adj_count: torch.Tensor,
                    budget_bytes: int, t_sample_ns: int, t_feature_ns: int, feat_policy: int = 0,
                    edge_count: Optional[torch.Tensor] = None, indices_rw: Optional[torch.Tensor] = None) -> Cache:
    """``indices_rw``: with DCI_FILL_ADJ_ELEMENTS the graph's own ``indices`` tensor, handed over as writable
    (the fill reorders the lists in place); defaults to ``graph.indices`` when that flag is set."""
    dev = ctx.device
    if feat_policy & DCI_FILL_ADJ_ELEMENTS:
        ctx.ensure_workspace(ctx.lib.dci_fill_elements_workspace_bytes(graph.num_nodes, graph.num_edges))
    else:
        ctx.ensure_workspace(ctx.lib.dci_fill_workspace_bytes(graph.num_nodes))
    total = (graph.num_nodes + 1 + graph.num_edges) * 8 + graph.num_nodes * graph.feat_dim * 4
    buf = torch.empty(min(int(budget_bytes), total) + 512, dtype=torch.uint8, device=dev)
    off = (-buf.data_ptr()) % 256
    adj_remap = torch.empty(graph.num_nodes, dtype=torch.int32, device=dev)
    feat_remap = torch.empty(graph.num_nodes, dtype=torch.int32, device=dev)
    c = _Cache()
    ctx.check(ctx.lib.dci_fill_caches(ctx.handle, C.byref(graph.c), _ptr(feat_count), _ptr(adj_count),
                                      _ptr(edge_count), int(budget_bytes), int(t_sample_ns), int(t_feature_ns),
                                      feat_policy, buf.data_ptr() + off, _ptr(adj_remap), _ptr(feat_remap),
                                      _ptr(indices_rw if indices_rw is not None else
                                           (graph.indices if feat_policy & DCI_FILL_ADJ_ELEMENTS else None)),
                                      C.byref(c)))
    cache = Cache(c, (buf, adj_remap, feat_remap))
    cache.adj_remap, cache.feat_remap, cache.buf, cache.buf_offset = adj_remap, feat_remap, buf, off
    return cache


def dci_sample_khop(ctx: Context, graph: Graph, cache: Optional[Cache], seeds: torch.Tensor, batch_index: int,
                    fanouts: Sequence[int], rng_seed: int, out: Blocks, stats: Optional[torch.Tensor] = None):
    assert seeds.is_cuda and seeds.dtype == torch.int64 and seeds.is_contiguous()
    ctx.ensure_workspace(ctx.lib.dci_sample_workspace_bytes(graph.num_nodes, seeds.numel(), _i32_array(fanouts), len(fanouts)))
    ctx.check(ctx.lib.dci_sample_khop(ctx.handle, C.byref(graph.c), None if cache is None else C.byref(cache.c),
                                      _ptr(seeds), seeds.numel(), batch_index, _i32_array(fanouts), len(fanouts),
                                      rng_seed, C.byref(out.c), _ptr(stats)))


STATIC_SCRATCH_BYTES = 32 << 20


def dci_sample_khop_static(ctx: Context, graph: Graph, cache: Optional[Cache], seeds: torch.Tensor, batch_index: int,
                           fanouts: Sequence[int], rng_seed: int, out: Blocks, stats: Optional[torch.Tensor] = None):
    """dci_sample_khop with the temporaries in the library's static device array: no workspace, no allocation."""
    assert seeds.is_cuda and seeds.dtype == torch.int64 and seeds.is_contiguous()
    ctx.check(ctx.lib.dci_sample_khop_static(ctx.handle, C.byref(graph.c), None if cache is None else C.byref(cache.c),
                                             _ptr(seeds), seeds.numel(), batch_index, _i32_array(fanouts),
                                             len(fanouts), rng_seed, C.byref(out.c), _ptr(stats)))


def dci_gather_features(ctx: Context, graph: Graph, cache: Optional[Cache], node_ids: torch.Tensor, n_max: int,
                        out: torch.Tensor, n_dev: Optional[int] = None, stats: Optional[torch.Tensor] = None):
    """``n_dev`` is the device address of an int64 row count (e.g. ``blocks.n_input_dev()``) or None."""
    assert node_ids.is_cuda and node_ids.dtype == torch.int64 and out.is_cuda and out.dtype == torch.float32
    assert out.numel() >= n_max * graph.feat_dim and node_ids.numel() >= n_max
    if stats is not None:
        ctx.ensure_workspace(1 << 20)
    ctx.check(ctx.lib.dci_gather_features(ctx.handle, C.byref(graph.c), None if cache is None else C.byref(cache.c),
                                          _ptr(node_ids), n_max, n_dev, _ptr(out), _ptr(stats)))


def dci_probe_read(ctx: Context, mem: torch.Tensor, granule: int, n_access: int = 0, order: int = 0,
                   workgroups: int = 4096, seed: int = 1, nbytes: Optional[int] = None) -> float:
    """GPU milliseconds of one probe kernel over ``mem`` (device or pinned host tensor); see dci_probe_read in dci.h."""
    assert mem.is_contiguous() and (mem.is_cuda or mem.is_pinned())
    total = mem.numel() * mem.element_size()
    base = mem.data_ptr()
    off = (-base) % 256
    nbytes = total - off if nbytes is None else min(int(nbytes), total - off)
    sink = torch.zeros(workgroups, dtype=torch.int64, device=ctx.device)
    ms = C.c_float(0.0)
    ctx.check(ctx.lib.dci_probe_read(ctx.handle, base + off, nbytes, granule, order, n_access, workgroups, seed,
                                     _ptr(sink), C.byref(ms)))
    return float(ms.value)


DCI_MODEL_SAGE_MEAN, DCI_MODEL_SAGE_SUM, DCI_MODEL_GCN_AVG = 0, 1, 2
DCI_FILL_STRICT_SPLIT, DCI_FILL_ADJ_ELEMENTS = 0x100, 0x200
DCI_OPT_LINEAR_KERNEL = 1
DCI_OPT_LINEAR_SPLIT = 2
DCI_OPT_RELABEL_SPIN_LIMIT = 3
DCI_OPT_TEST_RELABEL_FIRST_TICKET = 4
DCI_OPT_FUSED_INPUT = 5
DCI_OPT_RELABEL_TILE_ITERS = 6
DCI_OPT_INPUT_LAYER = 7


def dci_sage_forward(ctx: Context, blocks: Blocks, x_in: torch.Tensor, w_self: Sequence[torch.Tensor],
                     w_neigh: Sequence[torch.Tensor], bias: Sequence[torch.Tensor], logits: torch.Tensor):
    dci_gnn_forward(ctx, blocks, x_in, DCI_MODEL_SAGE_MEAN, w_self, w_neigh, bias, logits, _entry="dci_sage_forward")


def dci_gnn_forward(ctx: Context, blocks: Blocks, x_in: torch.Tensor, model: int,
                    w_self: Optional[Sequence[torch.Tensor]], w_neigh: Sequence[torch.Tensor],
                    bias: Sequence[torch.Tensor], logits: torch.Tensor, _entry: str = "dci_gnn_forward"):
    """``w_self`` may be None for DCI_MODEL_GCN_AVG (one weight matrix per layer)."""
    L = len(w_neigh)
    dims = [int(w_neigh[0].shape[0])] + [int(w.shape[1]) for w in w_neigh]
    for t in list(w_self or []) + list(w_neigh) + list(bias) + [x_in, logits]:
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
    assert logits.numel() >= blocks.cap_nodes[0] * dims[L]
    cap_rows = (C.c_int64 * DCI_MAX_HOPS)(*([blocks.cap_nodes[h] for h in range(L)] + [0] * (DCI_MAX_HOPS - L)))
    ctx.ensure_workspace(ctx.lib.dci_sage_workspace_bytes(cap_rows, L, _i32_array(dims)))
    arr = lambda ts: None if ts is None else (C.c_void_p * L)(*[t.data_ptr() for t in ts])
    if _entry == "dci_sage_forward":
        ctx.check(ctx.lib.dci_sage_forward(ctx.handle, C.byref(blocks.c), _ptr(x_in), L, _i32_array(dims), arr(w_self),
                                           arr(w_neigh), arr(bias), _ptr(logits)))
    else:
        ctx.check(ctx.lib.dci_gnn_forward(ctx.handle, C.byref(blocks.c), _ptr(x_in), L, _i32_array(dims), int(model),
                                          arr(w_self), arr(w_neigh), arr(bias), _ptr(logits)))


def dci_gather_forward(ctx: Context, graph: Graph, cache: Optional[Cache], blocks: Blocks, x: torch.Tensor, model: int,
                       w_self: Optional[Sequence[torch.Tensor]], w_neigh: Sequence[torch.Tensor],
                       bias: Sequence[torch.Tensor], logits: torch.Tensor, stats: Optional[torch.Tensor] = None):
    """Gather + forward with cached neighbour rows of the input layer read in place; ``x`` is scratch [cap_nodes, F]."""
    L = len(w_neigh)
    dims = [int(w_neigh[0].shape[0])] + [int(w.shape[1]) for w in w_neigh]
    for t in list(w_self or []) + list(w_neigh) + list(bias) + [x, logits]:
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
    assert x.numel() >= blocks.cap_nodes[L] * graph.feat_dim and logits.numel() >= blocks.cap_nodes[0] * dims[L]
    cap_rows = (C.c_int64 * DCI_MAX_HOPS)(*([blocks.cap_nodes[h] for h in range(L)] + [0] * (DCI_MAX_HOPS - L)))
    ctx.ensure_workspace(ctx.lib.dci_gather_forward_workspace_bytes(blocks.cap_nodes[L], cap_rows, L, _i32_array(dims)))
    arr = lambda ts: None if ts is None else (C.c_void_p * L)(*[t.data_ptr() for t in ts])
    ctx.check(ctx.lib.dci_gather_forward(ctx.handle, C.byref(graph.c), None if cache is None else C.byref(cache.c),
                                         C.byref(blocks.c), _ptr(x), L, _i32_array(dims), int(model), arr(w_self),
                                         arr(w_neigh), arr(bias), _ptr(logits), _ptr(stats)))


class Lane:
    """One lane of dci_infer_batches: a context on its own stream with its own batch buffers."""

    def __init__(self, graph: Graph, batch_size: int, fanouts: Sequence[int], dims: Sequence[int], device: int = 0,
                 stream: Optional["torch.cuda.Stream"] = None):
        self.stream = stream if stream is not None else torch.cuda.Stream(device)
        self.ctx = Context(device, stream=self.stream)
        self.blocks = Blocks(self.ctx, graph.num_nodes, batch_size, fanouts)
        self.x = torch.empty(max(self.blocks.cap_nodes[-1], 1), graph.feat_dim, dtype=torch.float32, device=self.ctx.device)
        L = len(fanouts)
        lib = self.ctx.lib
        cap_rows = (C.c_int64 * DCI_MAX_HOPS)(*([self.blocks.cap_nodes[h] for h in range(L)] + [0] * (DCI_MAX_HOPS - L)))
        need = max(lib.dci_sample_workspace_bytes(graph.num_nodes, batch_size, _i32_array(fanouts), L),
                   lib.dci_gather_forward_workspace_bytes(self.blocks.cap_nodes[L], cap_rows, L, _i32_array(dims)), 1 << 20)
        self.ctx.ensure_workspace(need)


def dci_infer_batches(lanes: Sequence[Lane], graph: Graph, cache: Optional[Cache], seeds: torch.Tensor, batch_size: int,
                      first_batch: int, n_batches: int, fanouts: Sequence[int], rng_seed: int, model: int,
                      w_self: Optional[Sequence[torch.Tensor]], w_neigh: Sequence[torch.Tensor],
                      bias: Sequence[torch.Tensor], logits: torch.Tensor, stats: Optional[torch.Tensor] = None):
    """Enqueues the batches round-robin on the lanes and returns; sync every lane's context before reading."""
    assert seeds.is_cuda and seeds.dtype == torch.int64 and seeds.is_contiguous()
    L = len(w_neigh)
    assert L == len(fanouts)
    dims = [int(w_neigh[0].shape[0])] + [int(w.shape[1]) for w in w_neigh]
    for t in list(w_self or []) + list(w_neigh) + list(bias) + [logits]:
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
    assert logits.numel() >= seeds.numel() * dims[L]
    arr = lambda ts: None if ts is None else (C.c_void_p * L)(*[t.data_ptr() for t in ts])
    c_lanes = (_Lane * len(lanes))()
    for k, ln in enumerate(lanes):
        c_lanes[k].ctx = ln.ctx.handle
        c_lanes[k].blocks = C.addressof(ln.blocks.c)
        c_lanes[k].x = ln.x.data_ptr()
    ctx = lanes[0].ctx
    ctx.check(ctx.lib.dci_infer_batches(c_lanes, len(lanes), C.byref(graph.c), None if cache is None else C.byref(cache.c),
                                        _ptr(seeds), seeds.numel(), batch_size, first_batch, n_batches,
                                        _i32_array(fanouts), L, rng_seed, int(model), _i32_array(dims), arr(w_self),
                                        arr(w_neigh), arr(bias), _ptr(logits), _ptr(stats)))
