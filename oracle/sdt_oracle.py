"""ctypes binding and step composition for the CPU oracle (sdt_oracle.c).

TEST INFRASTRUCTURE, NOT PRODUCT.  Only tests, the smoke check and the
benchmark's cpu_baseline leg import this module; the HIP package never does,
and this module never imports the HIP package or the input generator.

The step follows the per-worker loop the paper sketches in Sec. II-A and
Sec. III-D/E (sample a mini-batch sub-graph, fetch its features, aggregate
neighbourhoods in a GraphSAGE model, compute gradients, update the local
weights); the conventions the paper leaves open (fan-out order, frontier
order, bias/ReLU, plain SGD, bf16 storage points) are the ones stated in the
function docstrings below.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sdt_oracle.c")
_LIB_PATH = os.path.join(_HERE, "libsdt_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    if force or not os.path.exists(_LIB_PATH):
        subprocess.run(["gcc", "-O2", "-shared", "-fPIC", "-std=c11", _SRC, "-o", _LIB_PATH, "-lm"], check=True)
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
    L.orc_philox4x32_10.restype = None
    L.orc_philox4x32_10.argtypes = [vp, vp, vp]
    L.orc_sample_positions.restype = i32
    L.orc_sample_positions.argtypes = [i64, i32, u64, u32, u32, u32, vp]
    L.orc_sample_rows.restype = i64
    L.orc_sample_rows.argtypes = [vp, vp, vp, i32, i32, u64, u32, u32, vp, vp]
    L.orc_build_frontier.restype = i32
    L.orc_build_frontier.argtypes = [i64, vp, i32, vp, i64, vp, vp]
    L.orc_transpose_block.restype = None
    L.orc_transpose_block.argtypes = [i32, i32, vp, vp, vp, vp]
    L.orc_gather_rows.restype = None
    L.orc_gather_rows.argtypes = [vp, i64, i64, vp, i64, vp, i64]
    L.orc_aggregate_fwd.restype = None
    L.orc_aggregate_fwd.argtypes = [i64, vp, vp, vp, i64, vp]
    L.orc_linear_fwd.restype = None
    L.orc_linear_fwd.argtypes = [i64, i64, i64, vp, i64, vp, vp, vp, i32, vp]
    L.orc_softmax_xent.restype = f64
    L.orc_softmax_xent.argtypes = [i64, i64, vp, vp, vp]
    L.orc_linear_bwd.restype = None
    L.orc_linear_bwd.argtypes = [i64, i64, i64, vp, vp, i32, vp, i64, vp, vp, vp, vp, vp, vp]
    L.orc_gcn_aggregate_fwd.restype = None
    L.orc_gcn_aggregate_fwd.argtypes = [i64, vp, vp, vp, i64, vp, vp, vp, vp]
    L.orc_gcn_aggregate_bwd.restype = None
    L.orc_gcn_aggregate_bwd.argtypes = [i64, i64, vp, vp, vp, i64, vp, vp, vp, vp]
    L.orc_aggregate_bwd.restype = None
    L.orc_aggregate_bwd.argtypes = [i64, i64, vp, vp, vp, vp, i64, vp]
    L.orc_sgd.restype = None
    L.orc_sgd.argtypes = [i64, vp, vp, f64]
    L.orc_round_bf16.restype = None
    L.orc_round_bf16.argtypes = [i64, vp]
    _lib = L
    return L


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


# ------------------------------------------------------------------ primitives
def philox4x32_10(ctr, key) -> np.ndarray:
    c, k = _c(ctr, np.uint32), _c(key, np.uint32)
    out = np.empty(4, dtype=np.uint32)
    _load().orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def sample_positions(d: int, k: int, seed: int, step: int, layer: int, node: int) -> np.ndarray:
    pos = np.empty(max(k, 1), dtype=np.int64)
    m = _load().orc_sample_positions(d, k, seed, step, layer, node, _p(pos))
    return pos[:m].copy()


@dataclass
class Block:
    """One sampled bipartite layer.  src_nodes[:n_dst] are the destinations."""
    n_dst: int
    n_src: int
    indptr: np.ndarray     # int32 [n_dst+1]
    cols: np.ndarray       # int32 [nnz], local ids into src_nodes
    src_nodes: np.ndarray  # int32 [n_src], global ids
    e_glob: np.ndarray     # int32 [nnz], global ids of the sampled neighbours
    t_indptr: np.ndarray   # int32 [n_src+1]
    t_rows: np.ndarray     # int32 [nnz]

    @property
    def nnz(self) -> int:
        return int(self.indptr[-1])


def sample_block(indptr, indices, dst_nodes, fanout: int, seed: int, step: int, layer: int) -> Block:
    indptr, indices, dst = _c(indptr, np.int64), _c(indices, np.int32), _c(dst_nodes, np.int32)
    n_dst, n_nodes = len(dst), len(indptr) - 1
    b_indptr = np.zeros(n_dst + 1, dtype=np.int32)
    e_glob = np.empty(max(n_dst * max(fanout, 0), 1), dtype=np.int32)
    nnz = _load().orc_sample_rows(_p(indptr), _p(indices), _p(dst), n_dst, fanout, seed, step, layer,
                                  _p(b_indptr), _p(e_glob))
    e_glob = e_glob[:nnz].copy()
    src = np.empty(n_dst + nnz, dtype=np.int32)
    cols = np.empty(max(nnz, 1), dtype=np.int32)
    n_src = _load().orc_build_frontier(n_nodes, _p(dst), n_dst, _p(e_glob), nnz, _p(src), _p(cols))
    src, cols = src[:n_src].copy(), cols[:nnz].copy()
    t_indptr = np.zeros(n_src + 1, dtype=np.int32)
    t_rows = np.empty(max(nnz, 1), dtype=np.int32)
    _load().orc_transpose_block(n_dst, n_src, _p(b_indptr), _p(cols), _p(t_indptr), _p(t_rows))
    return Block(n_dst, n_src, b_indptr, cols, src, e_glob, t_indptr, t_rows[:nnz].copy())


def sample_blocks(indptr, indices, seeds, fanouts: List[int], seed: int, step: int) -> List[Block]:
    """blocks[l] feeds GNN layer l (l = 0 is the input-most layer and uses
    fanouts[0]).  Sampling starts at the seeds with the last fan-out and walks
    outwards; each block's source frontier is the next block's destinations."""
    L = len(fanouts)
    blocks: List[Optional[Block]] = [None] * L
    dst = _c(seeds, np.int32)
    for l in range(L - 1, -1, -1):
        blocks[l] = sample_block(indptr, indices, dst, fanouts[l], seed, step, l)
        dst = blocks[l].src_nodes
    return blocks


def gather_rows(X: np.ndarray, idx) -> np.ndarray:
    X = np.ascontiguousarray(X)
    idx = _c(idx, np.int32)
    out = np.empty((len(idx),) + X.shape[1:], dtype=X.dtype)
    rb = X.strides[0]
    _load().orc_gather_rows(_p(X), rb, rb, _p(idx), len(idx), _p(out), rb)
    return out


def aggregate_fwd(b_indptr, b_cols, H: np.ndarray, n_dst: Optional[int] = None) -> np.ndarray:
    ip, cols, H = _c(b_indptr, np.int64), _c(b_cols, np.int32), _c(H, np.float64)
    n_dst = len(ip) - 1 if n_dst is None else n_dst
    A = np.empty((n_dst, H.shape[1]), dtype=np.float64)
    _load().orc_aggregate_fwd(n_dst, _p(ip), _p(cols), _p(H), H.shape[1], _p(A))
    return A


def linear_fwd(Hself, A, W, b, relu: bool) -> np.ndarray:
    """Hself may have more rows than A; its first len(A) rows are used."""
    Hself, A, W, b = _c(Hself, np.float64), _c(A, np.float64), _c(W, np.float64), _c(b, np.float64)
    n, fin = A.shape
    fout = W.shape[1]
    assert W.shape[0] == 2 * fin and Hself.shape[1] == fin and Hself.shape[0] >= n
    Y = np.empty((n, fout), dtype=np.float64)
    _load().orc_linear_fwd(n, fin, fout, _p(Hself), fin, _p(A), _p(W), _p(b), int(relu), _p(Y))
    return Y


def softmax_xent(Z, y):
    Z, y = _c(Z, np.float64), _c(y, np.int32)
    dZ = np.empty_like(Z)
    loss = _load().orc_softmax_xent(Z.shape[0], Z.shape[1], _p(Z), _p(y), _p(dZ))
    return float(loss), dZ


def linear_bwd(dY, Y, relu: bool, Hself, A, W, need_input_grad: bool = True):
    dY, Y, Hself, A, W = (_c(x, np.float64) for x in (dY, Y, Hself, A, W))
    n, fin = A.shape
    fout = W.shape[1]
    dW = np.empty((2 * fin, fout), dtype=np.float64)
    db = np.empty(fout, dtype=np.float64)
    dSelf = np.empty((n, fin), dtype=np.float64) if need_input_grad else None
    dAgg = np.empty((n, fin), dtype=np.float64) if need_input_grad else None
    _load().orc_linear_bwd(n, fin, fout, _p(dY), _p(Y), int(relu), _p(Hself), fin, _p(A), _p(W),
                           _p(dW), _p(db), _p(dSelf), _p(dAgg))
    return dW, db, dSelf, dAgg


def aggregate_bwd(b_indptr, b_cols, n_src: int, dAgg, dSelf) -> np.ndarray:
    ip, cols, dAgg = _c(b_indptr, np.int64), _c(b_cols, np.int32), _c(dAgg, np.float64)
    dSelf = None if dSelf is None else _c(dSelf, np.float64)
    n_dst, F = dAgg.shape
    dH = np.empty((n_src, F), dtype=np.float64)
    _load().orc_aggregate_bwd(n_dst, n_src, _p(ip), _p(cols), _p(dAgg), _p(dSelf), F, _p(dH))
    return dH


def sgd(w, g, lr: float) -> np.ndarray:
    w = np.array(w, dtype=np.float64, copy=True, order="C")
    g = _c(g, np.float64)
    _load().orc_sgd(w.size, _p(w), _p(g), lr)
    return w


def round_bf16(x) -> np.ndarray:
    x = np.array(x, dtype=np.float64, copy=True, order="C")
    _load().orc_round_bf16(x.size, _p(x))
    return x


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float64."""
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ------------------------------------------------------------------ the step
def forward(blocks: List[Block], H0, W, b, bf16: bool = False):
    """Layer l: A = mean of sampled neighbours, Z = H[:n_dst] W_self + A W_neigh + b,
    ReLU on all but the last layer.  With bf16=True the tensors the bf16
    configuration stores in bf16 (A, hidden activations) are rounded when
    produced and the weights are rounded where they enter a product; logits
    stay unrounded."""
    rnd = round_bf16 if bf16 else (lambda t: t)
    L = len(blocks)
    H = [np.asarray(H0, dtype=np.float64)]
    A = []
    for l, blk in enumerate(blocks):
        a = rnd(aggregate_fwd(blk.indptr, blk.cols, H[l]))
        z = linear_fwd(H[l], a, rnd(W[l]), b[l], relu=(l < L - 1))
        A.append(a)
        H.append(rnd(z) if l < L - 1 else z)
    return H, A


def backward(blocks: List[Block], H, A, W, dZ, bf16: bool = False, relu_masks=None):
    """Gradients of every layer from the loss gradient dZ w.r.t. the logits.
    The ReLU derivative of hidden layer l is [H[l+1] > 0]; `relu_masks[l]`
    (boolean, same shape) replaces that decision when given -- the parity
    tests use it for pre-activations that sit within rounding of zero, where
    either decision is valid."""
    rnd = round_bf16 if bf16 else (lambda t: t)
    L = len(blocks)
    dH = rnd(dZ)
    dW, db = [None] * L, [None] * L
    dSelf, dAgg, dHs = [None] * L, [None] * L, [None] * L
    for l in range(L - 1, -1, -1):
        blk = blocks[l]
        Y = H[l + 1]
        if relu_masks is not None and l < L - 1 and relu_masks[l] is not None:
            Y = np.asarray(relu_masks[l], dtype=np.float64)
        dW[l], db[l], ds, da = linear_bwd(dH, Y, l < L - 1, H[l][:blk.n_dst], A[l], rnd(W[l]),
                                          need_input_grad=(l > 0))
        if l > 0:
            dSelf[l], dAgg[l] = rnd(ds), rnd(da)
            dH = rnd(aggregate_bwd(blk.indptr, blk.cols, blk.n_src, dAgg[l], dSelf[l]))
            dHs[l] = dH
    return dict(dW=dW, db=db, dSelf=dSelf, dAgg=dAgg, dH=dHs)


def train_step(indptr, indices, X, y, seeds, fanouts, W, b, seed: int, step: int, lr: float,
               bf16: bool = False, blocks: Optional[List[Block]] = None, relu_masks=None):
    """One mini-batch step.  X is fp32 (or uint16 bf16 bit patterns when
    bf16=True); W[l] is [2*in_l, out_l], b[l] is [out_l].  Returns a dict with
    every intermediate the HIP path can expose."""
    L = len(fanouts)
    if blocks is None:
        blocks = sample_blocks(indptr, indices, seeds, fanouts, seed, step)
    Xrows = gather_rows(X, blocks[0].src_nodes)
    H0 = bf16_bits_to_f64(Xrows) if bf16 else Xrows.astype(np.float64)
    W = [np.asarray(w, dtype=np.float64) for w in W]
    b = [np.asarray(v, dtype=np.float64) for v in b]
    H, A = forward(blocks, H0, W, b, bf16)
    loss, dZ = softmax_xent(H[L], np.asarray(y)[np.asarray(seeds)])
    g = backward(blocks, H, A, W, dZ, bf16, relu_masks)
    W_new = [sgd(W[l], g["dW"][l], lr) for l in range(L)]
    b_new = [sgd(b[l], g["db"][l], lr) for l in range(L)]
    return dict(blocks=blocks, H=H, A=A, logits=H[L], loss=loss, dZ=dZ, W=W, W_new=W_new, b_new=b_new, **g)


# ------------------------------------------------- beyond the mini-batch step
def infer_layerwise(indptr, indices, X, W, b, bf16: bool = False, kind: str = "sage", att=None,
                    slope: float = 0.2) -> np.ndarray:
    """Full-neighbour inference, one layer at a time over every node of the
    partition (the evaluation pass of Sec. IV-A: a trained model is scored on
    nodes with all of their neighbours, no sampling): for each layer,
    A = mean over the whole CSR row, H' = act(H W_self + A W_neigh + b), ReLU on
    all but the last layer.  Rounding points as in forward().  Returns the
    logits of all nodes in float64.
    kind = "gcn" / "gat": the same pass with the layer of gcn_train_step / gat_train_step, the block of
    a layer being the whole graph (every node a destination, its CSR row the edges, every neighbour
    kept, so the GCN weights are those of D~^-1/2 (Adj + I) D~^-1/2), and their rounding points."""
    rnd = round_bf16 if bf16 else (lambda t: t)
    H = bf16_bits_to_f64(np.asarray(X)) if bf16 else np.asarray(X, dtype=np.float64)
    L = len(W)
    ip = np.asarray(indptr, dtype=np.int64)
    cols = np.asarray(indices, dtype=np.int32)
    n = len(ip) - 1
    if kind == "gcn":
        s, c, selfw = gcn_weights(ip, np.arange(n), ip)
    for l in range(L):
        Wl, bl = np.asarray(W[l], dtype=np.float64), np.asarray(b[l], dtype=np.float64)
        if kind == "sage":
            a = rnd(aggregate_fwd(ip, cols, H))
            z = linear_fwd(H, a, rnd(Wl), bl, relu=(l < L - 1))
        elif kind == "gcn":
            a = rnd(gcn_aggregate_fwd(ip, cols, H, s, c, selfw))
            z = gcn_linear_fwd(a, rnd(Wl), bl, relu=(l < L - 1))
        elif kind == "gat":
            F = Wl.shape[1]
            a = np.asarray(att[l], dtype=np.float64)
            proj = rnd(H @ rnd(Wl))
            z = gat_aggregate_fwd(ip, cols, proj, a[:F], a[F:], slope)[0] + bl
            if l < L - 1:
                z = np.maximum(z, 0.0)
        else:
            raise ValueError(kind)
        H = rnd(z) if l < L - 1 else z
    return H


def model_average(params: List[np.ndarray], n_train: List[float]) -> np.ndarray:
    """Model synchronisation of Sec. III-D: w = sum_i alpha_i w_i with
    alpha_i = n_train_i / sum_j n_train_j (each worker's share of the training
    nodes), in float64."""
    tot = float(sum(n_train))
    out = np.zeros_like(np.asarray(params[0], dtype=np.float64))
    for p, n in zip(params, n_train):
        out = out + (float(n) / tot) * np.asarray(p, dtype=np.float64)
    return out


# ------------------------------------------------------------------ GCN (Sec. III-E: one of the integrated models)
def gcn_weights(indptr, src_nodes, b_indptr):
    """Edge and self weights of the GCN aggregation on a sampled block, from the degrees of
    the partition graph: with deg(v) the length of v's CSR row and m_i the number of sampled
    neighbours of destination i,
        c_j    = 1 / sqrt(deg(j) + 1)                    per source row j,
        s_i    = (deg(i) / m_i) / sqrt(deg(i) + 1)       per destination row i (0 if m_i = 0),
        self_i = 1 / (deg(i) + 1).
    A_i = s_i sum_e c_col h_col + self_i h_i is the sampled estimate of row i of
    D~^-1/2 (Adj + I) D~^-1/2 H with D~ = D + I; with every neighbour sampled (m_i = deg(i))
    it is that row exactly.  (The paper does not say how its GCN is normalised on sampled
    blocks; this is the reading used here.)"""
    ip = np.asarray(indptr, dtype=np.int64)
    src = np.asarray(src_nodes, dtype=np.int64)
    bip = np.asarray(b_indptr, dtype=np.int64)
    n_dst = len(bip) - 1
    deg = (ip[src + 1] - ip[src]).astype(np.float64)
    c = 1.0 / np.sqrt(deg + 1.0)
    m = np.diff(bip).astype(np.float64)
    d = deg[:n_dst]
    s = np.where(m > 0, (d / np.maximum(m, 1.0)) / np.sqrt(d + 1.0), 0.0)
    selfw = 1.0 / (d + 1.0)
    return s, c, selfw


def gcn_aggregate_fwd(b_indptr, b_cols, H, s, c, selfw) -> np.ndarray:
    ip, cols = _c(b_indptr, np.int64), _c(b_cols, np.int32)
    H = _c(H, np.float64)
    n_dst = len(ip) - 1
    A = np.zeros((n_dst, H.shape[1]), dtype=np.float64)
    s, c, selfw = _c(s, np.float64), _c(c, np.float64), _c(selfw, np.float64)
    _load().orc_gcn_aggregate_fwd(n_dst, _p(ip), _p(cols), _p(H), H.shape[1], _p(s), _p(c), _p(selfw), _p(A))
    return A


def gcn_aggregate_bwd(b_indptr, b_cols, n_src: int, dA, s, c, selfw) -> np.ndarray:
    ip, cols = _c(b_indptr, np.int64), _c(b_cols, np.int32)
    dA = _c(dA, np.float64)
    n_dst, F = len(ip) - 1, dA.shape[1]
    dH = np.zeros((n_src, F), dtype=np.float64)
    s, c, selfw = _c(s, np.float64), _c(c, np.float64), _c(selfw, np.float64)
    _load().orc_gcn_aggregate_bwd(n_dst, n_src, _p(ip), _p(cols), _p(dA), F, _p(s), _p(c), _p(selfw), _p(dH))
    return dH


def gcn_linear_fwd(A, W, b, relu: bool) -> np.ndarray:
    """Z = A W + b with W [in, out] (one weight matrix, no separate self operand)."""
    Z = np.asarray(A, dtype=np.float64) @ np.asarray(W, dtype=np.float64) + np.asarray(b, dtype=np.float64)
    return np.maximum(Z, 0.0) if relu else Z


def gcn_train_step(indptr, indices, X, y, seeds, fanouts, W, b, seed: int, step: int, lr: float,
                   blocks: Optional[List[Block]] = None, relu_masks=None, bf16: bool = False):
    """One mini-batch step of a GCN: layer l is H' = act(Agcn(H) W_l + b_l), W_l [in_l, out_l], ReLU on
    all but the last layer; sampling, loss and SGD as in train_step.  With bf16=True X holds bf16 bit
    patterns (uint16) and the rounding points are those of forward() / backward(): the aggregated rows,
    the hidden activations and the gradients w.r.t. both are rounded when produced, the weights and the
    loss gradient where they enter a product; logits, loss, dW, db are not rounded."""
    rnd = round_bf16 if bf16 else (lambda t: t)
    L = len(fanouts)
    if blocks is None:
        blocks = sample_blocks(indptr, indices, seeds, fanouts, seed, step)
    Xrows = gather_rows(X, blocks[0].src_nodes)
    H = [bf16_bits_to_f64(Xrows) if bf16 else Xrows.astype(np.float64)]
    W = [np.asarray(w, dtype=np.float64) for w in W]
    b = [np.asarray(v, dtype=np.float64) for v in b]
    A, wts = [], []
    for l, blk in enumerate(blocks):
        wt = gcn_weights(indptr, blk.src_nodes, blk.indptr)
        a = rnd(gcn_aggregate_fwd(blk.indptr, blk.cols, H[l], *wt))
        A.append(a)
        wts.append(wt)
        z = gcn_linear_fwd(a, rnd(W[l]), b[l], relu=(l < L - 1))
        H.append(rnd(z) if l < L - 1 else z)
    loss, dZ = softmax_xent(H[L], np.asarray(y)[np.asarray(seeds)])
    dW, db, dA, dHs = [None] * L, [None] * L, [None] * L, [None] * L
    dY = rnd(dZ)
    for l in range(L - 1, -1, -1):
        blk = blocks[l]
        if l < L - 1:
            keep = H[l + 1] > 0
            if relu_masks is not None and relu_masks[l] is not None:
                keep = np.asarray(relu_masks[l], dtype=bool)
            dY = dY * keep
        dW[l] = A[l].T @ dY
        db[l] = dY.sum(axis=0)
        if l > 0:
            dA[l] = rnd(dY @ rnd(W[l]).T)
            dY = rnd(gcn_aggregate_bwd(blk.indptr, blk.cols, blk.n_src, dA[l], *wts[l]))
            dHs[l] = dY
    W_new = [sgd(W[l], dW[l], lr) for l in range(L)]
    b_new = [sgd(b[l], db[l], lr) for l in range(L)]
    return dict(blocks=blocks, H=H, A=A, logits=H[L], loss=loss, dZ=dZ, W=W, W_new=W_new, b_new=b_new, dW=dW, db=db,
                dA=dA, dH=dHs, weights=wts)


# ------------------------------------------------------------------ Adam
def adam(w, g, m, v, t: int, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8):
    """One Adam update (Kingma & Ba) in float64: m <- b1 m + (1-b1) g, v <- b2 v + (1-b2) g^2,
    w <- w - lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps); t counts updates from 1.
    Returns (w, m, v).  (The paper does not name its optimiser; plain SGD is the default here.)"""
    w, g = np.asarray(w, dtype=np.float64), np.asarray(g, dtype=np.float64)
    m = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    return w - lr * mhat / (np.sqrt(vhat) + eps), m, v


# ------------------------------------------------------------------ GAT attention aggregation (Sec. III-E: GAT is one of the integrated models)
def _leaky(x, slope):
    return np.where(x > 0, x, slope * x)


def gat_aggregate_fwd(b_indptr, b_cols, z, a_src, a_dst, slope: float = 0.2):
    """Single-head graph attention over a sampled block (Velickovic et al.), on already projected
    features z [n_src, F] (row i < n_dst is destination i itself):
        s_(i<-j) = LeakyReLU(a_dst . z_i + a_src . z_j),   j over row i's edges and j = i (a self edge,
        so that no softmax is empty), alpha = softmax over that set, out_i = sum alpha_(i<-j) z_j.
    Returns (out [n_dst, F], alpha per edge [nnz], alpha of the self edge [n_dst]).  float64.
    (The paper does not describe its GAT variant; one head, slope 0.2 and the self edge are this
    build's reading.)"""
    ip = np.asarray(b_indptr, dtype=np.int64)
    cols = np.asarray(b_cols, dtype=np.int64)
    z = np.asarray(z, dtype=np.float64)
    a_src, a_dst = np.asarray(a_src, dtype=np.float64), np.asarray(a_dst, dtype=np.float64)
    n_dst = len(ip) - 1
    el, er = z @ a_src, z[:n_dst] @ a_dst
    out = np.zeros((n_dst, z.shape[1]))
    alpha, alpha_self = np.zeros(len(cols)), np.zeros(n_dst)
    for i in range(n_dst):
        c = cols[ip[i]:ip[i + 1]]
        s = _leaky(er[i] + np.concatenate([el[c], el[i:i + 1]]), slope)
        p = np.exp(s - s.max())
        a = p / p.sum()
        alpha[ip[i]:ip[i + 1]], alpha_self[i] = a[:-1], a[-1]
        out[i] = a[:-1] @ z[c] + a[-1] * z[i]
    return out, alpha, alpha_self


def gat_aggregate_bwd(b_indptr, b_cols, z, a_src, a_dst, g, slope: float = 0.2):
    """Gradients of gat_aggregate_fwd's output w.r.t. z, a_src, a_dst given g = d loss / d out [n_dst, F]."""
    ip = np.asarray(b_indptr, dtype=np.int64)
    cols = np.asarray(b_cols, dtype=np.int64)
    z, g = np.asarray(z, dtype=np.float64), np.asarray(g, dtype=np.float64)
    a_src, a_dst = np.asarray(a_src, dtype=np.float64), np.asarray(a_dst, dtype=np.float64)
    n_dst = len(ip) - 1
    _, alpha, alpha_self = gat_aggregate_fwd(ip, cols, z, a_src, a_dst, slope)
    el, er = z @ a_src, z[:n_dst] @ a_dst
    dz = np.zeros_like(z)
    d_el, d_er = np.zeros(z.shape[0]), np.zeros(n_dst)
    for i in range(n_dst):
        c = np.concatenate([cols[ip[i]:ip[i + 1]], [i]])
        a = np.concatenate([alpha[ip[i]:ip[i + 1]], alpha_self[i:i + 1]])
        d_alpha = z[c] @ g[i]                          # d out_i / d alpha_e = z_col
        np.add.at(dz, c, a[:, None] * g[i][None, :])   # through the weighted sum
        d_s = a * (d_alpha - a @ d_alpha)              # softmax
        pre = er[i] + el[c]
        d_pre = d_s * np.where(pre > 0, 1.0, slope)    # LeakyReLU
        d_er[i] = d_pre.sum()
        np.add.at(d_el, c, d_pre)
    dz += d_el[:, None] * a_src[None, :]
    dz[:n_dst] += d_er[:, None] * a_dst[None, :]
    return dz, z.T @ d_el, z[:n_dst].T @ d_er


def gat_train_step(indptr, indices, X, y, seeds, fanouts, W, b, att, seed: int, step: int, lr: float,
                   slope: float = 0.2, blocks: Optional[List[Block]] = None, relu_masks=None, bf16: bool = False):
    """One mini-batch step of a single-head GAT (Sec. III-E names GAT as an integrated model and
    Sec. III-C as the most expensive one; the variant is not described).  Layer l projects EVERY
    frontier row, z = H_l W_l (W_l [in_l, out_l], no bias inside the attention), aggregates with
    gat_aggregate_fwd using att[l] = [a_src | a_dst] (2 out_l values), adds b_l and applies ReLU on
    all but the last layer; sampling, loss and SGD as in train_step.  With bf16=True X holds bf16 bit
    patterns (uint16) and what is stored between kernels is rounded when produced: the projected rows z,
    the hidden activations and the gradients w.r.t. both; the weights are rounded where they enter a
    matrix product; the attention vectors and scalars, the logits, the loss gradient (it enters no matrix
    product here), dW, db and datt are not rounded."""
    rnd = round_bf16 if bf16 else (lambda t: t)
    L = len(fanouts)
    if blocks is None:
        blocks = sample_blocks(indptr, indices, seeds, fanouts, seed, step)
    Xrows = gather_rows(X, blocks[0].src_nodes)
    H = [bf16_bits_to_f64(Xrows) if bf16 else Xrows.astype(np.float64)]
    W = [np.asarray(w, dtype=np.float64) for w in W]
    b = [np.asarray(v, dtype=np.float64) for v in b]
    att = [np.asarray(v, dtype=np.float64) for v in att]
    Z = []
    for l, blk in enumerate(blocks):
        F = W[l].shape[1]
        z = rnd(H[l] @ rnd(W[l]))
        out, _, _ = gat_aggregate_fwd(blk.indptr, blk.cols, z, att[l][:F], att[l][F:], slope)
        pre = out + b[l]
        Z.append(z)
        H.append(rnd(np.maximum(pre, 0.0)) if l < L - 1 else pre)
    loss, dZ = softmax_xent(H[L], np.asarray(y)[np.asarray(seeds)])
    dW, db, datt, dz, dHs = [None] * L, [None] * L, [None] * L, [None] * L, [None] * L
    g = dZ
    for l in range(L - 1, -1, -1):
        blk = blocks[l]
        F = W[l].shape[1]
        if l < L - 1:
            keep = H[l + 1] > 0
            if relu_masks is not None and relu_masks[l] is not None:
                keep = np.asarray(relu_masks[l], dtype=bool)
            g = g * keep
        db[l] = g.sum(axis=0)
        dz[l], da_src, da_dst = gat_aggregate_bwd(blk.indptr, blk.cols, Z[l], att[l][:F], att[l][F:], g, slope)
        dz[l] = rnd(dz[l])
        datt[l] = np.concatenate([da_src, da_dst])
        dW[l] = H[l].T @ dz[l]
        if l > 0:
            g = rnd(dz[l] @ rnd(W[l]).T)
            dHs[l] = g
    W_new = [sgd(W[l], dW[l], lr) for l in range(L)]
    b_new = [sgd(b[l], db[l], lr) for l in range(L)]
    att_new = [sgd(att[l], datt[l], lr) for l in range(L)]
    return dict(blocks=blocks, H=H, Z=Z, logits=H[L], loss=loss, dZ=dZ, W=W, W_new=W_new, b_new=b_new, att_new=att_new,
                dW=dW, db=db, datt=datt, dz=dz, dH=dHs)
