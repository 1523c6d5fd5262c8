"""Seeded synthetic inputs (graphs, features, seed nodes, weights) and the workload table.

Input generators only: nothing here samples, counts, fills a cache, gathers or runs a
model.  Both the CPU oracle's tests and the GPU path's tests draw their inputs from this
module so that they see identical bytes.  The native part is ``dci_synth.cpp`` (plain
C++, host only), loaded through ctypes; arrays are numpy, or any buffer whose address is
passed with ``ptr=`` (for example pinned host tensors).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dci_synth.cpp")
_LIB = os.environ.get("DCI_SYNTH_LIB") or os.path.join(_HERE, "libdci_synth.so")  # override: the sanitizer build
_lib = None


def build(force: bool = False) -> str:
    """Compile the generator library with g++ (host code only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def build_sanitized() -> str:
    """The generator library with AddressSanitizer and UndefinedBehaviorSanitizer (DCI_SYNTH_LIB selects it)."""
    out = os.path.join(_HERE, "libdci_synth_asan.so")
    cmd = ["g++", "-std=c++17", "-fPIC", "-shared", "-pthread", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1", "-o", out, _SRC]
    subprocess.run(cmd, check=True)
    return out


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        lib = ctypes.CDLL(_LIB)
        c = ctypes
        lib.synth_rmat_csr.argtypes = [c.c_int64, c.c_int64, c.c_double, c.c_double, c.c_double,
                                       c.c_uint64, c.c_void_p, c.c_void_p, c.c_int32]
        lib.synth_rmat_csr.restype = c.c_int32
        lib.synth_features.argtypes = [c.c_int64, c.c_int32, c.c_uint64, c.c_void_p, c.c_int32]
        lib.synth_features.restype = c.c_int32
        lib.synth_seeds.argtypes = [c.c_int64, c.c_int64, c.c_uint64, c.c_void_p]
        lib.synth_seeds.restype = c.c_int32
        lib.synth_glorot.argtypes = [c.c_int64, c.c_int64, c.c_uint64, c.c_uint64, c.c_void_p]
        lib.synth_glorot.restype = c.c_int32
        lib.synth_uniform.argtypes = [c.c_int64, c.c_double, c.c_uint64, c.c_uint64, c.c_void_p]
        lib.synth_uniform.restype = c.c_int32
        _lib = lib
    return _lib


def default_threads() -> int:
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        return int(env)
    return max(1, min(16, os.cpu_count() or 1))


# --------------------------------------------------------------------------------------
# workload table


@dataclass(frozen=True)
class Workload:
    """One benchmark / parity configuration.

    ``fanouts`` are in execution order from the seed nodes outward (the reverse of the
    layer-ordered lists such as "15,10,5" that the paper prints).
    """
    name: str
    num_nodes: int
    num_edges: int
    feat_dim: int
    fanouts: Tuple[int, ...]
    num_seeds: int
    batch_size: int
    hidden: int
    classes: int
    budget_bytes: int
    rmat: Tuple[float, float, float] = (0.57, 0.19, 0.19)
    graph_seed: int = 1
    feature_seed: int = 2
    seed_seed: int = 3
    rng_seed: int = 4
    weight_seed: int = 5
    n_presample: int = 8
    presample_first_batch: int = 1 << 31

    @property
    def n_hops(self) -> int:
        return len(self.fanouts)

    @property
    def adj_bytes(self) -> int:
        return (self.num_nodes + 1 + self.num_edges) * 8

    @property
    def feat_bytes(self) -> int:
        return self.num_nodes * self.feat_dim * 4

    @property
    def dims(self) -> Tuple[int, ...]:
        return (self.feat_dim,) + (self.hidden,) * (self.n_hops - 1) + (self.classes,)

    @property
    def num_batches(self) -> int:
        return (self.num_seeds + self.batch_size - 1) // self.batch_size

    def cap_nodes(self, n_seeds: Optional[int] = None) -> List[int]:
        """Upper bound on |F_h| for h = 0..L with ``n_seeds`` seeds in the batch."""
        b = self.batch_size if n_seeds is None else n_seeds
        caps = [b]
        for f in self.fanouts:
            caps.append(min(self.num_nodes, caps[-1] * (1 + f)))
        return caps

    def cap_edges(self, n_seeds: Optional[int] = None) -> List[int]:
        caps = self.cap_nodes(n_seeds)
        return [caps[h] * f for h, f in enumerate(self.fanouts)]

    def scaled(self, name: str, **kw) -> "Workload":
        return replace(self, name=name, **kw)


_TINY_BYTES = (16384 + 1 + 163840) * 8 + 16384 * 64 * 4

WORKLOADS: Dict[str, Workload] = {
    w.name: w
    for w in [
        Workload("tiny", 16_384, 163_840, 64, (5, 10), 2_048, 256, 64, 16, _TINY_BYTES // 5),
        Workload("medium", 232_965, 114_600_000, 602, (5, 10, 15), 55_000, 1_024, 256, 41, 4_000_000_000),
        Workload("large", 2_449_029, 61_900_000, 100, (5, 10, 15), 200_000, 4_096, 256, 47, 2_000_000_000),
        Workload("huge", 111_059_956, 1_615_685_872, 128, (5, 10, 15), 1_000_000, 4_096, 256, 172,
                 64_000_000_000),
        Workload("skewed", 65_000_000, 1_800_000_000, 256, (10, 25), 500_000, 8_192, 256, 64,
                 48_000_000_000, rmat=(0.65, 0.15, 0.15)),
        # the paper's two other datasets by shape (Table II), with the three-layer, hidden-128 models of
        # Table III; run with the sum-aggregate GraphSAGE or the GCN of dci_gnn_forward
        Workload("yelp", 716_480, 6_977_410, 300, (5, 10, 15), 100_000, 4_096, 128, 100, 1_000_000_000),
        Workload("amazon", 1_598_960, 132_169_734, 200, (5, 10, 15), 200_000, 4_096, 128, 107, 2_000_000_000),
    ]
}


# --------------------------------------------------------------------------------------
# generators


def _addr(arr: Optional[np.ndarray], ptr: Optional[int]) -> int:
    return int(ptr) if ptr is not None else arr.ctypes.data


def rmat_csr(num_nodes: int, num_edges: int, rmat=(0.57, 0.19, 0.19), seed: int = 1, *,
             indptr_ptr: Optional[int] = None, indices_ptr: Optional[int] = None,
             threads: Optional[int] = None):
    """R-MAT multigraph as int64 CSR by destination (each list sorted ascending).

    Without ``*_ptr`` returns ``(indptr, indices)`` numpy arrays; with them writes into the
    caller's buffers (``(N+1)*8`` and ``E*8`` bytes) and returns ``None``.
    """
    lib = _load()
    own = indptr_ptr is None
    if own:
        indptr = np.empty(num_nodes + 1, dtype=np.int64)
        indices = np.empty(max(num_edges, 1), dtype=np.int64)[:num_edges]
        indptr_ptr, indices_ptr = indptr.ctypes.data, indices.ctypes.data
    rc = lib.synth_rmat_csr(num_nodes, num_edges, rmat[0], rmat[1], rmat[2], seed,
                            indptr_ptr, indices_ptr, threads or default_threads())
    if rc != 0:
        raise ValueError("synth_rmat_csr: bad arguments")
    return (indptr, indices) if own else None


def features(num_nodes: int, feat_dim: int, seed: int = 2, *, ptr: Optional[int] = None,
             threads: Optional[int] = None):
    lib = _load()
    out = None
    if ptr is None:
        out = np.empty((num_nodes, feat_dim), dtype=np.float32)
    rc = lib.synth_features(num_nodes, feat_dim, seed, _addr(out, ptr), threads or default_threads())
    if rc != 0:
        raise ValueError("synth_features: bad arguments")
    return out


def seeds(num_nodes: int, num_seeds: int, seed: int = 3) -> np.ndarray:
    lib = _load()
    out = np.empty(num_seeds, dtype=np.int64)
    if lib.synth_seeds(num_nodes, num_seeds, seed, out.ctypes.data) != 0:
        raise ValueError("synth_seeds: bad arguments")
    return out


def sage_weights(dims, seed: int = 5):
    """Glorot-uniform ``W_self``/``W_neigh`` [d_in, d_out] and a small uniform bias per layer."""
    lib = _load()
    w_self, w_neigh, bias = [], [], []
    for layer in range(len(dims) - 1):
        di, do = int(dims[layer]), int(dims[layer + 1])
        ws = np.empty((di, do), dtype=np.float32)
        wn = np.empty((di, do), dtype=np.float32)
        b = np.empty(do, dtype=np.float32)
        lib.synth_glorot(di, do, seed, 3 * layer + 0, ws.ctypes.data)
        lib.synth_glorot(di, do, seed, 3 * layer + 1, wn.ctypes.data)
        lib.synth_uniform(do, 0.1, seed, 3 * layer + 2, b.ctypes.data)
        w_self.append(ws)
        w_neigh.append(wn)
        bias.append(b)
    return w_self, w_neigh, bias


def make_inputs(w: Workload, with_features: bool = True):
    """All host-side inputs of one workload as numpy arrays (small and medium sizes)."""
    indptr, indices = rmat_csr(w.num_nodes, w.num_edges, w.rmat, w.graph_seed)
    feat = features(w.num_nodes, w.feat_dim, w.feature_seed) if with_features else None
    sd = seeds(w.num_nodes, w.num_seeds, w.seed_seed)
    ws, wn, b = sage_weights(w.dims, w.weight_seed)
    return dict(indptr=indptr, indices=indices, feat=feat, seeds=sd, w_self=ws, w_neigh=wn, bias=b)
