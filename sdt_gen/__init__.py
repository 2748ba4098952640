"""Seeded synthetic inputs for the per-worker GraphSAGE step (host only).

Thin ctypes binding over ``gen.cpp`` plus the five workload recipes.  The
module serves the CPU oracle's tests and the HIP path's tests/bench alike and
contains none of the method's arithmetic; it imports neither of them.

The graphs stand in for the public datasets of the paper's Table "Dataset
statistics": same node/edge scale, feature width and class count, power-law
degrees; nothing of the datasets themselves is reproduced.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "gen.cpp"), os.path.join(_HERE, "spring.cpp")]
_LIB_PATH = os.path.join(_HERE, "libsdt_gen.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile gen.cpp and spring.cpp into libsdt_gen.so next to them."""
    if force or not os.path.exists(_LIB_PATH):
        cmd = ["g++", "-O3", "-fopenmp", "-shared", "-fPIC", "-std=c++17", *_SRCS, "-o", _LIB_PATH]
        subprocess.run(cmd, check=True)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        build(force=True)
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, u32, u64, f64 = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64,
                                   ctypes.c_uint32, ctypes.c_uint64, ctypes.c_double)
    L.sdtgen_rmat.restype = vp
    L.sdtgen_rmat.argtypes = [i32, i64, f64, f64, f64, u64]
    L.sdtgen_chunglu.restype = vp
    L.sdtgen_chunglu.argtypes = [i64, i64, f64, f64, u64]
    L.sdtgen_csr_nodes.restype = i64
    L.sdtgen_csr_nodes.argtypes = [vp]
    L.sdtgen_csr_nnz.restype = i64
    L.sdtgen_csr_nnz.argtypes = [vp]
    L.sdtgen_csr_copy.restype = None
    L.sdtgen_csr_copy.argtypes = [vp, vp, vp]
    L.sdtgen_csr_free.restype = None
    L.sdtgen_csr_free.argtypes = [vp]
    L.sdtgen_normal_f32.restype = None
    L.sdtgen_normal_f32.argtypes = [vp, i64, u64, u32]
    L.sdtgen_normal_bf16.restype = None
    L.sdtgen_normal_bf16.argtypes = [vp, i64, u64, u32]
    L.sdtgen_labels.restype = None
    L.sdtgen_labels.argtypes = [vp, i64, i32, u64]
    L.sdtgen_uniform_f32.restype = None
    L.sdtgen_uniform_f32.argtypes = [vp, i64, ctypes.c_float, u64, u32]
    L.sdtgen_seed_batch.restype = i32
    L.sdtgen_seed_batch.argtypes = [vp, i32, i32, i32, u64, u32]
    L.sdtgen_edge_count.restype = i64
    L.sdtgen_edge_count.argtypes = [i64, vp, vp]
    L.sdtgen_edge_stream.restype = None
    L.sdtgen_edge_stream.argtypes = [i64, vp, vp, u64, vp, vp]
    L.sdtgen_spring.restype = vp
    L.sdtgen_spring.argtypes = [i64, vp, vp, vp, i64, i32, f64, i64]
    L.sdtgen_spring_clusters.restype = i64
    L.sdtgen_spring_clusters.argtypes = [vp, i32]
    L.sdtgen_spring_copy.restype = None
    L.sdtgen_spring_copy.argtypes = [vp, vp, vp, vp]
    L.sdtgen_spring_free.restype = None
    L.sdtgen_spring_free.argtypes = [vp]
    L.sdtgen_partition.restype = vp
    L.sdtgen_partition.argtypes = [i64, vp, vp, vp, i32]
    for name in ("nodes", "owned", "nnz"):
        getattr(L, "sdtgen_partition_" + name).restype = i64
        getattr(L, "sdtgen_partition_" + name).argtypes = [vp]
    L.sdtgen_partition_copy.restype = None
    L.sdtgen_partition_copy.argtypes = [vp, vp, vp, vp]
    L.sdtgen_partition_free.restype = None
    L.sdtgen_partition_free.argtypes = [vp]
    _lib = L
    return L


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _take_csr(h):
    L = _load()
    n, nnz = L.sdtgen_csr_nodes(h), L.sdtgen_csr_nnz(h)
    indptr = np.empty(n + 1, dtype=np.int64)
    indices = np.empty(nnz, dtype=np.int32)
    L.sdtgen_csr_copy(h, _ptr(indptr), _ptr(indices))
    L.sdtgen_csr_free(h)
    return indptr, indices


def rmat_csr(log2n: int, n_pairs: int, seed: int, a=0.57, b=0.19, c=0.19):
    """Symmetric, sorted, duplicate-free CSR of an R-MAT graph with 2**log2n nodes."""
    return _take_csr(_load().sdtgen_rmat(log2n, n_pairs, a, b, c, seed))


def chunglu_csr(n: int, n_pairs: int, avg_deg: float, gamma: float, seed: int):
    """Symmetric, sorted, duplicate-free CSR of a Chung-Lu power-law graph."""
    return _take_csr(_load().sdtgen_chunglu(n, n_pairs, avg_deg, gamma, seed))


def normal_features(n: int, f: int, seed: int, bf16: bool = False, stream: int = 0) -> np.ndarray:
    """[n, f] N(0,1) features; fp32, or bf16 bit patterns as uint16."""
    if bf16:
        out = np.empty((n, f), dtype=np.uint16)
        _load().sdtgen_normal_bf16(_ptr(out), n * f, seed, stream)
    else:
        out = np.empty((n, f), dtype=np.float32)
        _load().sdtgen_normal_f32(_ptr(out), n * f, seed, stream)
    return out


def labels(n: int, n_classes: int, seed: int) -> np.ndarray:
    out = np.empty(n, dtype=np.int32)
    _load().sdtgen_labels(_ptr(out), n, n_classes, seed)
    return out


def glorot_sage_weights(dims: List[int], seed: int):
    """Per layer l: W[l] = [W_self; W_neigh] of shape [2*in, out], each half
    U(-a, a) with a = sqrt(6/(in+out)); b[l] = 0."""
    Ws, bs = [], []
    for l in range(len(dims) - 1):
        fi, fo = dims[l], dims[l + 1]
        W = np.empty((2 * fi, fo), dtype=np.float32)
        _load().sdtgen_uniform_f32(_ptr(W), W.size, math.sqrt(6.0 / (fi + fo)), seed, l)
        Ws.append(W)
        bs.append(np.zeros(fo, dtype=np.float32))
    return Ws, bs


def seed_batch(batch: int, lo: int, hi: int, seed: int, step: int) -> np.ndarray:
    """`batch` distinct node ids drawn uniformly from [lo, hi) for one mini-batch."""
    out = np.empty(batch, dtype=np.int32)
    rc = _load().sdtgen_seed_batch(_ptr(out), batch, lo, hi, seed, step)
    if rc != 0:
        raise ValueError("seed range smaller than the batch")
    return out


# --------------------------------------------------------------------------
# Partitions with replicas (the paper's streaming partitioner as a workload producer)
# --------------------------------------------------------------------------
def edge_stream(indptr: np.ndarray, indices: np.ndarray, order_seed: int = 1):
    """Every undirected edge of a symmetric CSR once, as two int32 arrays (u, v): in row order with
    u < v when order_seed is 0, else in a seeded random order with a random orientation."""
    L, n = _load(), len(indptr) - 1
    m = L.sdtgen_edge_count(n, _ptr(indptr), _ptr(indices))
    eu, ev = np.empty(m, dtype=np.int32), np.empty(m, dtype=np.int32)
    L.sdtgen_edge_stream(n, _ptr(indptr), _ptr(indices), order_seed, _ptr(eu), _ptr(ev))
    return eu, ev


def spring(indptr: np.ndarray, indices: np.ndarray, p: int, beta: float = 1.05, tau_vol: Optional[int] = None,
           order_seed: int = 1, stream=None) -> dict:
    """Algorithm 1 of the paper over the edge stream of a symmetric CSR.  tau_vol defaults to the
    graph's volume over p (the paper names the threshold without giving its value).  Returns
    part / cluster_stream / cluster_merged (int32 [n]) and the two cluster counts."""
    L, n = _load(), len(indptr) - 1
    degree = np.ascontiguousarray(np.diff(indptr).astype(np.int64))
    eu, ev = stream if stream is not None else edge_stream(indptr, indices, order_seed)
    eu, ev = np.ascontiguousarray(eu, dtype=np.int32), np.ascontiguousarray(ev, dtype=np.int32)
    if tau_vol is None:
        tau_vol = int(degree.sum()) // p
    h = L.sdtgen_spring(n, _ptr(degree), _ptr(eu), _ptr(ev), len(eu), p, beta, tau_vol)
    out = {k: np.empty(n, dtype=np.int32) for k in ("part", "cluster_stream", "cluster_merged")}
    L.sdtgen_spring_copy(h, _ptr(out["part"]), _ptr(out["cluster_stream"]), _ptr(out["cluster_merged"]))
    out["n_clusters_stream"], out["n_clusters_merged"] = L.sdtgen_spring_clusters(h, 0), L.sdtgen_spring_clusters(h, 1)
    L.sdtgen_spring_free(h)
    return out


def partition_csr(indptr: np.ndarray, indices: np.ndarray, part: np.ndarray, which: int):
    """The edge pass for one partition: (local indptr int64, local indices int32, global_id int32,
    n_owned).  Local ids: owned nodes in ascending global id, then replicas in ascending global id;
    an owned row keeps its full neighbour list, a replica's row only its owned neighbours."""
    L, n = _load(), len(indptr) - 1
    part = np.ascontiguousarray(part, dtype=np.int32)
    h = L.sdtgen_partition(n, _ptr(indptr), _ptr(indices), _ptr(part), which)
    nl, nnz = L.sdtgen_partition_nodes(h), L.sdtgen_partition_nnz(h)
    lp, li, gid = np.empty(nl + 1, dtype=np.int64), np.empty(nnz, dtype=np.int32), np.empty(nl, dtype=np.int32)
    L.sdtgen_partition_copy(h, _ptr(lp), _ptr(li), _ptr(gid))
    n_owned = L.sdtgen_partition_owned(h)
    L.sdtgen_partition_free(h)
    return lp, li, gid, int(n_owned)


# --------------------------------------------------------------------------
# Workload recipes
# --------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    kind: str                 # "rmat" | "chunglu"
    log2n: int
    avg_deg: float
    feat: int
    classes: int
    hidden: int
    layers: int
    fanouts: List[int]        # input-most layer first
    batch: int
    seed: int
    steps: int
    owned_frac: float = 1.0   # seeds are drawn from the first owned_frac * N ids
    bf16: bool = False
    directed_then_sym: bool = False
    gamma: float = 2.1
    dims: List[int] = field(default_factory=list)

    def __post_init__(self):
        if not self.dims:
            self.dims = [self.feat] + [self.hidden] * (self.layers - 1) + [self.classes]

    @property
    def n_nodes(self) -> int:
        return 1 << self.log2n


WORKLOADS = {
    # 2-layer model on a small R-MAT graph; the case the oracle finishes in seconds.
    "tiny": Workload("tiny", "rmat", 14, 16, 64, 8, 64, 2, [10, 5], 256, 0, 1, owned_frac=0.5),
    # one of four partitions of a products-sized graph (deg ~25, F=100, C=47)
    "products": Workload("products", "rmat", 21, 25, 100, 47, 256, 2, [15, 10], 1024, 1, 100, owned_frac=0.25),
    # reddit-sized dense neighbourhoods (deg ~490, F=602, C=41)
    "dense": Workload("dense", "chunglu", 18, 490, 602, 41, 256, 2, [25, 10], 1024, 2, 100),
    # papers-partition-sized sparse graph, bf16 storage, 3 layers
    "sparse_bf16": Workload("sparse_bf16", "rmat", 24, 15, 128, 172, 256, 3, [15, 10, 5], 1024, 3, 200,
                            bf16=True, directed_then_sym=True),
    # full-neighbour single layer over all nodes (no sampling); dims = [256, 256]
    "fullgraph": Workload("fullgraph", "rmat", 22, 32, 256, 256, 256, 1, [], 0, 4, 1, dims=[256, 256]),
}


@dataclass
class Instance:
    wl: Workload
    indptr: np.ndarray        # int64 [N+1]
    indices: np.ndarray       # int32 [nnz]
    X: Optional[np.ndarray]   # [N, F] fp32, or uint16 bf16 bit patterns
    y: Optional[np.ndarray]   # int32 [N]
    W: list
    b: list
    n_owned: Optional[int] = None          # a partition with replicas: local ids [0, n_owned) are owned
    global_id: Optional[np.ndarray] = None  # ... and local id i is node global_id[i] of the partitioned graph
    info: Optional[dict] = None

    @property
    def n_nodes(self) -> int:
        return len(self.indptr) - 1

    @property
    def seed_range(self):
        if self.n_owned is not None:
            return 0, self.n_owned
        return 0, max(self.wl.batch, int(self.wl.n_nodes * self.wl.owned_frac))

    def batch(self, step: int) -> np.ndarray:
        lo, hi = self.seed_range
        return seed_batch(self.wl.batch, lo, hi, self.wl.seed, step)


def make_graph(wl: Workload):
    n = wl.n_nodes
    if wl.kind == "rmat":
        # "average degree d" counts CSR entries per node after both directions
        # are stored: d*N/2 pairs, or d*N directed draws when the recipe says
        # the graph is generated directed and then symmetrised.
        pairs = int(n * wl.avg_deg) if wl.directed_then_sym else int(n * wl.avg_deg / 2)
        return rmat_csr(wl.log2n, pairs, wl.seed)
    if wl.kind == "chunglu":
        return chunglu_csr(n, int(n * wl.avg_deg / 2), wl.avg_deg, wl.gamma, wl.seed)
    raise ValueError(wl.kind)


def make_instance(wl: Workload, with_features: bool = True) -> Instance:
    indptr, indices = make_graph(wl)
    X = normal_features(wl.n_nodes, wl.feat, wl.seed, bf16=wl.bf16) if with_features else None
    y = labels(wl.n_nodes, wl.classes, wl.seed) if with_features else None
    W, b = glorot_sage_weights(wl.dims, wl.seed)
    return Instance(wl, indptr, indices, X, y, W, b)


def drop_isolated(indptr: np.ndarray, indices: np.ndarray):
    """The same graph without its degree-0 nodes, the others renumbered in ascending order."""
    deg = np.diff(indptr)
    keep = deg > 0
    new = np.cumsum(keep) - 1
    out_ptr = np.concatenate([[0], np.cumsum(deg[keep])]).astype(np.int64)
    return out_ptr, new[indices].astype(np.int32)


def make_partition_instance(wl: Workload, p: int = 4, which: int = 0, beta: float = 1.05, order_seed: int = 1,
                            with_features: bool = True) -> Instance:
    """One worker's partition as the paper's partitioner produces it: the workload's graph without
    its isolated nodes (the public graphs have next to none; R-MAT leaves many) goes through
    Algorithm 1 with p partitions, and partition `which` comes back as a local graph: owned nodes
    first, replicas of their outside neighbours after them, features and labels those of the
    global nodes.  Mini-batch seeds are drawn from the owned nodes only."""
    indptr, indices = drop_isolated(*make_graph(wl))
    n = len(indptr) - 1
    sp = spring(indptr, indices, p, beta=beta, order_seed=order_seed)
    lp, li, gid, n_owned = partition_csr(indptr, indices, sp["part"], which)
    X = y = None
    if with_features:
        X = np.ascontiguousarray(normal_features(n, wl.feat, wl.seed, bf16=wl.bf16)[gid])
        y = np.ascontiguousarray(labels(n, wl.classes, wl.seed)[gid])
    W, b = glorot_sage_weights(wl.dims, wl.seed)
    loads = np.bincount(sp["part"], minlength=p)
    info = dict(p=p, which=which, beta=beta, n_global=n, n_local=len(gid), n_owned=n_owned, nnz_local=int(lp[-1]),
                owned_per_partition=loads.tolist(), n_clusters_stream=int(sp["n_clusters_stream"]),
                n_clusters_merged=int(sp["n_clusters_merged"]))
    return Instance(wl, lp, li, X, y, W, b, n_owned=n_owned, global_id=gid, info=info)
