"""Thin ctypes binding over libsdt.so: argument marshalling only.

Every function has the name of the C entry point it calls (see include/sdt.h),
takes torch tensors that already live on the GPU, passes their device pointers
and the current torch stream, and raises SdtError when the library reports a
failure.  Nothing is computed here; there is no fallback: if libsdt.so is
missing the import of the library fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsdt.so")

SDT_OK, SDT_ERR_INVALID_ARG, SDT_ERR_WORKSPACE, SDT_ERR_HIP = 0, -1, -2, -3
SDT_F32, SDT_BF16 = 0, 1
SDT_MAX_LAYERS = 8
SDT_MAX_FANOUT = 64
SDT_MODEL_SAGE_MEAN, SDT_MODEL_GCN, SDT_MODEL_GAT = 0, 1, 2
SDT_OPT_SGD, SDT_OPT_ADAM = 0, 1

_vp, _i32, _i64, _u32, _u64, _sz = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32,
                                    ctypes.c_uint64, ctypes.c_size_t)


class SdtError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"sdt error {code}: {msg}")
        self.code = code


class sdt_csr(ctypes.Structure):
    _fields_ = [("n_nodes", _i64), ("indptr", _vp), ("indices", _vp)]


class sdt_block(ctypes.Structure):
    _fields_ = [("cap_dst", _i32), ("cap_src", _i32), ("cap_nnz", _i32), ("reserved", _i32),
                ("counts", _vp), ("indptr", _vp), ("cols", _vp), ("src_nodes", _vp),
                ("t_indptr", _vp), ("t_rows", _vp)]


class sdt_model(ctypes.Structure):
    _fields_ = [("n_layers", _i32), ("dims", _i32 * (SDT_MAX_LAYERS + 1)),
                ("W", _vp * SDT_MAX_LAYERS), ("b", _vp * SDT_MAX_LAYERS),
                ("dW", _vp * SDT_MAX_LAYERS), ("db", _vp * SDT_MAX_LAYERS), ("kind", _i32), ("optimizer", _i32),
                ("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float), ("gat_slope", ctypes.c_float),
                ("mW", _vp * SDT_MAX_LAYERS), ("vW", _vp * SDT_MAX_LAYERS), ("mb", _vp * SDT_MAX_LAYERS),
                ("vb", _vp * SDT_MAX_LAYERS), ("att", _vp * SDT_MAX_LAYERS), ("datt", _vp * SDT_MAX_LAYERS),
                ("matt", _vp * SDT_MAX_LAYERS), ("vatt", _vp * SDT_MAX_LAYERS)]


class sdt_step_layout(ctypes.Structure):
    _L = SDT_MAX_LAYERS
    _fields_ = [("total_bytes", _u64), ("header", _u64), ("state", _u64), ("n_layers", _i32),
                ("cap_dst", _i32 * _L), ("cap_src", _i32 * _L), ("cap_nnz", _i32 * _L),
                ("counts", _u64 * _L), ("indptr", _u64 * _L), ("cols", _u64 * _L), ("src_nodes", _u64 * _L),
                ("t_indptr", _u64 * _L), ("t_rows", _u64 * _L),
                ("H", _u64 * (_L + 1)), ("A", _u64 * _L), ("dZ", _u64),
                ("dH", _u64 * _L), ("dSelf", _u64 * _L), ("dAgg", _u64 * _L),
                ("dW", _u64 * _L), ("db", _u64 * _L), ("row_loss", _u64), ("scratch", _u64), ("wlow", _u64), ("norm", _u64 * _L),
                ("z", _u64 * _L), ("dz", _u64 * _L), ("datt", _u64 * _L), ("gatws", _u64 * _L), ("ld_in", _u64)]


class sdt_partition(ctypes.Structure):
    _fields_ = [("graph", sdt_csr), ("X", _vp), ("ldx", _i64), ("labels", _vp), ("seeds", _vp),
                ("n_steps", _i32), ("reserved", _i32), ("n_train", _i64)]


EXPORTS = {
    "sdt_version": (ctypes.c_char_p, []),
    "sdt_last_error": (ctypes.c_char_p, []),
    "sdt_struct_bytes": (_sz, [_i32]),
    "sdt_sample_workspace_bytes": (_sz, [_i64, _i32, _i32]),
    "sdt_sample_csr": (_i32, [_vp, _vp, _i32, _vp, _i32, _u64, _u32, _u32, _vp, _vp, _sz, _vp]),
    "sdt_gather_features": (_i32, [_vp, _i64, _i32, _i32, _vp, _i32, _vp, _vp, _i64, _vp]),
    "sdt_sage_aggregate_fwd": (_i32, [_vp, _vp, _i64, _i32, _i32, _vp, _i64, _vp]),
    "sdt_sage_aggregate_csr_fwd": (_i32, [_vp, _vp, _i64, _i32, _i32, _vp, _i64, _vp]),
    "sdt_sage_layer_csr_fused_ok": (_i32, [_i32, _i32, _i32]),
    "sdt_sage_layer_csr_fwd": (_i32, [_vp, _vp, _i64, _i32, _i32, _vp, _vp, _i32, _i32, _vp, _i64, _vp]),
    "sdt_sage_aggregate_gather_fwd": (_i32, [_vp, _vp, _i64, _i32, _i32, _vp, _i64, _vp]),
    "sdt_sage_aggregate_bwd": (_i32, [_vp, _vp, _i64, _vp, _i64, _vp, _i32, _i32, _vp, _i64, _vp]),
    "sdt_sage_linear_fwd": (_i32, [_vp, _i64, _vp, _i64, _i32, _vp, _i32, _i32, _vp, _vp, _i32, _i32, _vp, _i64,
                                   _i32, _vp]),
    "sdt_linear_bwd_workspace_bytes": (_sz, [_i32, _i32, _i32]),
    "sdt_sage_linear_bwd": (_i32, [_vp, _i64, _i32, _vp, _i64, _i32, _vp, _i64, _vp, _i64, _i32, _vp, _i32, _i32,
                                   _vp, _i32, _vp, _vp, _vp, _vp, _i64, _vp, _sz, _vp]),
    "sdt_sage_linear_bwd_noalloc": (_i32, [_vp, _i64, _i32, _vp, _i64, _i32, _vp, _i64, _vp, _i64, _i32, _vp, _i32, _i32,
                                           _vp, _i32, _vp, _vp, _vp, _vp, _i64, _vp]),
    "sdt_train_step_layout": (_i32, [_i64, _i32, _vp, _vp, _i32, _vp]),
    "sdt_train_step": (_i32, [_vp, _vp, _i64, _i32, _vp, _vp, _i32, _vp, _vp, _u64, _u32, ctypes.c_float, _vp, _vp,
                              _vp, _sz, _vp]),
    "sdt_train_loop_workspace_bytes": (_sz, [_i64, _i32, _vp, _vp, _i32]),
    "sdt_train_loop": (_i32, [_vp, _vp, _i64, _i32, _vp, _vp, _i32, _i32, _vp, _vp, _u64, _u32, ctypes.c_float, _vp,
                              _vp, _vp, _sz, _vp, _vp, _i32]),
    "sdt_gcn_norm": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp]),
    "sdt_gcn_aggregate_fwd": (_i32, [_vp, _vp, _i64, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _i64, _vp]),
    "sdt_gcn_aggregate_bwd": (_i32, [_vp, _vp, _i64, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _i64, _vp]),
    "sdt_gat_workspace_bytes": (_sz, [_i32, _i32, _i32]),
    "sdt_gat_aggregate_fwd": (_i32, [_vp, _vp, _i64, _i32, _i32, _vp, _vp, ctypes.c_float, _vp, _i64, _vp, _sz, _vp]),
    "sdt_gat_aggregate_bwd": (_i32, [_vp, _vp, _i64, _i32, _i32, _vp, _vp, ctypes.c_float, _vp, _i64, _vp, _i64, _vp, _vp,
                                     _vp, _sz, _vp]),
    "sdt_infer_layerwise_workspace_bytes": (_sz, [_i64, _vp, _i32]),
    "sdt_infer_layerwise": (_i32, [_vp, _vp, _i64, _i32, _vp, _vp, _i64, _vp, _sz, _vp]),
    "sdt_model_average": (_i32, [_vp, _vp, _i32, _i64, _vp, _vp]),
    "sdt_train_round_workspace_bytes": (_sz, [_vp, _i32, _i32, _vp, _vp, _i32]),
    "sdt_train_round": (_i32, [_vp, _i32, _i32, _i32, _vp, _vp, _vp, _u64, _u32, ctypes.c_float, _vp, _vp, _sz, _vp,
                               _vp, _i32]),
    "sdt_timing_create": (_i32, [_i32, _u64, _vp]),
    "sdt_timing_create_wide": (_i32, [_i32, _vp, _vp]),
    "sdt_timing_destroy": (None, [_vp]),
    "sdt_timing_reset": (None, [_vp]),
    "sdt_timing_set_stride": (_i32, [_vp, _i32]),
    "sdt_timing_read": (_i32, [_vp, _i32, _i32, _vp, _vp]),
}

STAGES = {"sample": 0, "gather": 1, "aggregate_fwd": 2, "linear_fwd": 3, "loss": 4, "linear_bwd": 5,
          "aggregate_bwd": 6, "head": 7, "sample_rows": 8, "front_scan": 9, "front_apply": 10, "relabel": 11,
          "transpose": 12, "update": 13, "bwd_weight": 14, "bwd_input": 15}
SDT_STAGE_MASK_WORDS = 2

_lib = None


def lib() -> ctypes.CDLL:
    """Load libsdt.so (built by paper_2404_02300_amd.build); no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(there is no CPU or PyTorch fallback for the HIP path)")
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _check(rc: int):
    if rc != SDT_OK:
        raise SdtError(rc, lib().sdt_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda, "device tensor expected"
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SDT_F32
    if t.dtype == torch.bfloat16:
        return SDT_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def sdt_version() -> str:
    return lib().sdt_version().decode()


def sdt_last_error() -> str:
    return lib().sdt_last_error().decode()


def sdt_struct_bytes(which: int) -> int:
    return int(lib().sdt_struct_bytes(which))


# ----------------------------------------------------------------- graph / block holders
class Csr:
    """Device CSR (int64 indptr, int32 indices) plus its C struct."""

    def __init__(self, indptr: torch.Tensor, indices: torch.Tensor):
        assert indptr.dtype == torch.int64 and indices.dtype == torch.int32 and indptr.is_cuda and indices.is_cuda
        self.indptr, self.indices = indptr.contiguous(), indices.contiguous()
        self.n_nodes = indptr.numel() - 1
        self.c = sdt_csr(self.n_nodes, self.indptr.data_ptr(), self.indices.data_ptr())


class Block:
    """Caller-owned device arrays of one sampled layer plus the C struct."""

    def __init__(self, cap_dst: int, fanout: int, n_nodes: int, device, transposed: bool = True):
        cap_nnz = cap_dst * fanout
        cap_src = max(cap_dst, min(cap_dst + cap_nnz, n_nodes))
        i32 = dict(dtype=torch.int32, device=device)
        self.cap_dst, self.cap_src, self.cap_nnz = cap_dst, cap_src, cap_nnz
        self.counts = torch.zeros(4, **i32)
        self.indptr = torch.zeros(cap_dst + 1, **i32)
        self.cols = torch.zeros(max(cap_nnz, 1), **i32)
        self.src_nodes = torch.zeros(max(cap_src, 1), **i32)
        self.t_indptr = torch.zeros(cap_src + 1, **i32) if transposed else None
        self.t_rows = torch.zeros(max(cap_nnz, 1), **i32) if transposed else None
        self.c = sdt_block(cap_dst, cap_src, cap_nnz, 0, self.counts.data_ptr(), self.indptr.data_ptr(),
                           self.cols.data_ptr(), self.src_nodes.data_ptr(),
                           self.t_indptr.data_ptr() if transposed else None,
                           self.t_rows.data_ptr() if transposed else None)

    @classmethod
    def from_arrays(cls, indptr, cols, n_src: int, src_nodes=None, t_indptr=None, t_rows=None):
        """Wrap existing device arrays (e.g. an oracle-built block uploaded for a unit test)."""
        self = cls.__new__(cls)
        dev = indptr.device
        n_dst, nnz = indptr.numel() - 1, cols.numel()
        self.cap_dst, self.cap_src, self.cap_nnz = n_dst, n_src, nnz
        self.counts = torch.tensor([n_dst, n_src, nnz, 0], dtype=torch.int32, device=dev)
        self.indptr, self.cols = indptr, cols
        self.src_nodes, self.t_indptr, self.t_rows = src_nodes, t_indptr, t_rows
        self.c = sdt_block(n_dst, n_src, nnz, 0, self.counts.data_ptr(), indptr.data_ptr(),
                           cols.data_ptr() if nnz else None,
                           src_nodes.data_ptr() if src_nodes is not None else None,
                           t_indptr.data_ptr() if t_indptr is not None else None,
                           t_rows.data_ptr() if t_rows is not None and nnz else None)
        return self


# ----------------------------------------------------------------- entry points
def sdt_sample_workspace_bytes(n_nodes: int, cap_dst: int, fanout: int) -> int:
    return lib().sdt_sample_workspace_bytes(n_nodes, cap_dst, fanout)


def sdt_sample_csr(graph: Csr, dst_nodes: torch.Tensor, fanout: int, seed: int, step: int, layer: int, out: Block,
                   ws: torch.Tensor, n_dst_d: Optional[torch.Tensor] = None, n_dst_cap: Optional[int] = None):
    cap = dst_nodes.numel() if n_dst_cap is None else n_dst_cap
    _check(lib().sdt_sample_csr(ctypes.byref(graph.c), _ptr(dst_nodes) if dst_nodes.numel() else None, cap,
                                _ptr(n_dst_d), fanout, seed, step, layer, ctypes.byref(out.c), _ptr(ws),
                                ws.numel() * ws.element_size(), _stream()))


def sdt_gather_features(X: torch.Tensor, idx: torch.Tensor, out: torch.Tensor, n_d: Optional[torch.Tensor] = None):
    _check(lib().sdt_gather_features(_ptr(X), X.stride(0), X.shape[1], dtype_code(X), _ptr(idx), idx.numel(),
                                     _ptr(n_d), _ptr(out), out.stride(0), _stream()))


def sdt_sage_aggregate_fwd(blk: Block, H: torch.Tensor, A: torch.Tensor):
    _check(lib().sdt_sage_aggregate_fwd(ctypes.byref(blk.c), _ptr(H), H.stride(0), H.shape[1], dtype_code(H),
                                        _ptr(A), A.stride(0), _stream()))


def sdt_sage_aggregate_gather_fwd(blk: Block, X: torch.Tensor, A: torch.Tensor):
    _check(lib().sdt_sage_aggregate_gather_fwd(ctypes.byref(blk.c), _ptr(X), X.stride(0), X.shape[1], dtype_code(X),
                                               _ptr(A), A.stride(0), _stream()))


def sdt_sage_aggregate_csr_fwd(graph: Csr, H: torch.Tensor, A: torch.Tensor):
    _check(lib().sdt_sage_aggregate_csr_fwd(ctypes.byref(graph.c), _ptr(H), H.stride(0), H.shape[1], dtype_code(H),
                                            _ptr(A), A.stride(0), _stream()))


def sdt_sage_layer_csr_fused_ok(fin: int, fout: int, dtype: int) -> bool:
    return bool(lib().sdt_sage_layer_csr_fused_ok(fin, fout, dtype))


def sdt_sage_layer_csr_fwd(graph: Csr, H: torch.Tensor, W: torch.Tensor, b: Optional[torch.Tensor], relu: bool,
                           Y: torch.Tensor):
    """One full-neighbour layer over the whole graph in one launch: Y = act([H | mean_nbr(H)] W + b)."""
    _check(lib().sdt_sage_layer_csr_fwd(ctypes.byref(graph.c), _ptr(H), H.stride(0), H.shape[1], W.shape[1], _ptr(W),
                                        _ptr(b), int(relu), dtype_code(H), _ptr(Y), Y.stride(0), _stream()))


def sdt_sage_aggregate_bwd(blk: Block, dAgg: torch.Tensor, dSelf: Optional[torch.Tensor], dH: torch.Tensor,
                           relu_of: Optional[torch.Tensor] = None):
    _check(lib().sdt_sage_aggregate_bwd(ctypes.byref(blk.c), _ptr(dAgg), dAgg.stride(0), _ptr(dSelf),
                                        dSelf.stride(0) if dSelf is not None else 0, _ptr(relu_of), dAgg.shape[1],
                                        dtype_code(dAgg), _ptr(dH), dH.stride(0), _stream()))


def sdt_sage_linear_fwd(Hself: torch.Tensor, A: torch.Tensor, W: torch.Tensor, b: torch.Tensor, relu: bool,
                        Y: torch.Tensor, n_d: Optional[torch.Tensor] = None):
    n, fin = A.shape
    _check(lib().sdt_sage_linear_fwd(_ptr(Hself), Hself.stride(0), _ptr(A), A.stride(0), n, _ptr(n_d), fin,
                                     W.shape[1], _ptr(W), _ptr(b), int(relu), dtype_code(A), _ptr(Y), Y.stride(0),
                                     dtype_code(Y), _stream()))


def sdt_linear_bwd_workspace_bytes(n_cap: int, fin: int, fout: int) -> int:
    return lib().sdt_linear_bwd_workspace_bytes(n_cap, fin, fout)


def sdt_sage_linear_bwd(dY: torch.Tensor, Y: Optional[torch.Tensor], relu: bool, Hself: torch.Tensor,
                        A: torch.Tensor, W: torch.Tensor, dW: torch.Tensor, db: torch.Tensor,
                        dSelf: Optional[torch.Tensor], dAgg: Optional[torch.Tensor], ws: torch.Tensor,
                        n_d: Optional[torch.Tensor] = None):
    n, fin = A.shape
    _check(lib().sdt_sage_linear_bwd(_ptr(dY), dY.stride(0), dtype_code(dY), _ptr(Y),
                                     Y.stride(0) if Y is not None else 0, int(relu), _ptr(Hself), Hself.stride(0),
                                     _ptr(A), A.stride(0), n, _ptr(n_d), fin, W.shape[1], _ptr(W), dtype_code(A),
                                     _ptr(dW), _ptr(db), _ptr(dSelf), _ptr(dAgg),
                                     dSelf.stride(0) if dSelf is not None else 0, _ptr(ws),
                                     ws.numel() * ws.element_size(), _stream()))


SDT_NOALLOC_SCRATCH_BYTES = 32 << 20


def sdt_sage_linear_bwd_noalloc(dY: torch.Tensor, Y: Optional[torch.Tensor], relu: bool, Hself: torch.Tensor,
                                A: torch.Tensor, W: torch.Tensor, dW: torch.Tensor, db: torch.Tensor,
                                dSelf: Optional[torch.Tensor], dAgg: Optional[torch.Tensor],
                                n_d: Optional[torch.Tensor] = None):
    """sdt_sage_linear_bwd with the library's built-in scratch: no workspace argument."""
    n, fin = A.shape
    _check(lib().sdt_sage_linear_bwd_noalloc(_ptr(dY), dY.stride(0), dtype_code(dY), _ptr(Y),
                                             Y.stride(0) if Y is not None else 0, int(relu), _ptr(Hself),
                                             Hself.stride(0), _ptr(A), A.stride(0), n, _ptr(n_d), fin, W.shape[1],
                                             _ptr(W), dtype_code(A), _ptr(dW), _ptr(db), _ptr(dSelf), _ptr(dAgg),
                                             dSelf.stride(0) if dSelf is not None else 0, _stream()))


def make_model(dims: Sequence[int], W: List[torch.Tensor], b: List[torch.Tensor],
               dW: Optional[List[torch.Tensor]] = None, db: Optional[List[torch.Tensor]] = None,
               kind: int = SDT_MODEL_SAGE_MEAN, att: Optional[List[torch.Tensor]] = None,
               datt: Optional[List[torch.Tensor]] = None, gat_slope: float = 0.2) -> sdt_model:
    """GAT (kind = SDT_MODEL_GAT) also takes att[l], fp32 [2 * dims[l+1]] = [a_src | a_dst]."""
    m = sdt_model()
    m.kind = kind
    m.gat_slope = gat_slope
    m.n_layers = len(dims) - 1
    for i, d in enumerate(dims):
        m.dims[i] = d
    for l in range(m.n_layers):
        rows = 2 * dims[l] if kind == SDT_MODEL_SAGE_MEAN else dims[l]
        assert W[l].dtype == torch.float32 and W[l].is_contiguous() and tuple(W[l].shape) == (rows, dims[l + 1])
        m.W[l], m.b[l] = W[l].data_ptr(), b[l].data_ptr()
        m.dW[l] = dW[l].data_ptr() if dW is not None else None
        m.db[l] = db[l].data_ptr() if db is not None else None
        if kind == SDT_MODEL_GAT:
            assert att is not None and att[l].dtype == torch.float32 and att[l].is_contiguous() and att[l].numel() == 2 * dims[l + 1]
            m.att[l] = att[l].data_ptr()
            m.datt[l] = datt[l].data_ptr() if datt is not None else None
    return m


def use_adam(model: sdt_model, mW: List[torch.Tensor], vW: List[torch.Tensor], mb: List[torch.Tensor],
             vb: List[torch.Tensor], beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
             matt: Optional[List[torch.Tensor]] = None, vatt: Optional[List[torch.Tensor]] = None) -> sdt_model:
    """Switch a model to Adam; the moment tensors (fp32, shaped like W / b, zero before the first step)
    stay owned by the caller."""
    model.optimizer, model.beta1, model.beta2, model.eps = SDT_OPT_ADAM, beta1, beta2, eps
    for l in range(model.n_layers):
        for t in (mW[l], vW[l], mb[l], vb[l]):
            assert t.dtype == torch.float32 and t.is_contiguous()
        model.mW[l], model.vW[l], model.mb[l], model.vb[l] = (mW[l].data_ptr(), vW[l].data_ptr(), mb[l].data_ptr(),
                                                              vb[l].data_ptr())
        if matt is not None:
            model.matt[l], model.vatt[l] = matt[l].data_ptr(), vatt[l].data_ptr()
    return model


def sdt_train_step_layout(n_nodes: int, batch: int, fanouts: Sequence[int], model: sdt_model,
                          dtype: int) -> sdt_step_layout:
    lay = sdt_step_layout()
    f = (_i32 * len(fanouts))(*fanouts)
    _check(lib().sdt_train_step_layout(n_nodes, batch, f, ctypes.byref(model), dtype, ctypes.byref(lay)))
    return lay


def sdt_train_step(graph: Csr, X: torch.Tensor, labels: torch.Tensor, seeds: torch.Tensor, fanouts: Sequence[int],
                   model: sdt_model, seed: int, step: int, lr: float, loss: torch.Tensor, ws: torch.Tensor,
                   timing: Optional["Timing"] = None):
    f = (_i32 * len(fanouts))(*fanouts)
    _check(lib().sdt_train_step(ctypes.byref(graph.c), _ptr(X), X.stride(0), dtype_code(X), _ptr(labels),
                                _ptr(seeds), seeds.numel(), f, ctypes.byref(model), seed, step, lr, _ptr(loss),
                                timing.handle if timing is not None else None,
                                _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def sdt_train_loop_workspace_bytes(n_nodes: int, batch: int, fanouts: Sequence[int], model: sdt_model,
                                   dtype: int) -> int:
    f = (_i32 * len(fanouts))(*fanouts)
    return lib().sdt_train_loop_workspace_bytes(n_nodes, batch, f, ctypes.byref(model), dtype)


def _aux_array(aux_streams):
    """None, one torch stream or a sequence of them -> (host array of stream handles, count)."""
    if aux_streams is None:
        return None, 0
    if isinstance(aux_streams, torch.cuda.Stream):
        aux_streams = [aux_streams]
    return (_vp * len(aux_streams))(*[s.cuda_stream for s in aux_streams]), len(aux_streams)


def sdt_train_loop(graph: Csr, X: torch.Tensor, labels: torch.Tensor, seeds: torch.Tensor, fanouts: Sequence[int],
                   model: sdt_model, seed: int, first_step: int, lr: float, losses: torch.Tensor, ws: torch.Tensor,
                   aux_streams=None, timing: Optional["Timing"] = None):
    """seeds: int32 [n_steps, batch] on the device; losses: fp32 [n_steps]; aux_streams: None (serial),
    one torch stream or up to three."""
    assert seeds.dim() == 2 and seeds.is_contiguous() and losses.numel() >= seeds.shape[0]
    f = (_i32 * len(fanouts))(*fanouts)
    main = _stream()
    aux, n_aux = _aux_array(aux_streams)
    _check(lib().sdt_train_loop(ctypes.byref(graph.c), _ptr(X), X.stride(0), dtype_code(X), _ptr(labels),
                                _ptr(seeds), seeds.shape[1], seeds.shape[0], f, ctypes.byref(model), seed,
                                first_step, lr, _ptr(losses), timing.handle if timing is not None else None,
                                _ptr(ws), ws.numel() * ws.element_size(), main, aux, n_aux))


def sdt_gcn_norm(graph: Csr, blk: Block, c: torch.Tensor, s: torch.Tensor, selfw: torch.Tensor):
    _check(lib().sdt_gcn_norm(ctypes.byref(graph.c), ctypes.byref(blk.c), _ptr(c), _ptr(s), _ptr(selfw), _stream()))


def sdt_gcn_aggregate_fwd(blk: Block, H: torch.Tensor, c: torch.Tensor, s: torch.Tensor, selfw: torch.Tensor,
                          A: torch.Tensor, through_src_nodes: bool = False):
    _check(lib().sdt_gcn_aggregate_fwd(ctypes.byref(blk.c), _ptr(H), H.stride(0), int(through_src_nodes), H.shape[1],
                                       dtype_code(H), _ptr(c), _ptr(s), _ptr(selfw), _ptr(A), A.stride(0), _stream()))


def sdt_gcn_aggregate_bwd(blk: Block, dA: torch.Tensor, c: torch.Tensor, s: torch.Tensor, selfw: torch.Tensor,
                          dH: torch.Tensor, relu_of: Optional[torch.Tensor] = None):
    _check(lib().sdt_gcn_aggregate_bwd(ctypes.byref(blk.c), _ptr(dA), dA.stride(0),
                                       _ptr(relu_of) if relu_of is not None else None, dA.shape[1], dtype_code(dA),
                                       _ptr(c), _ptr(s), _ptr(selfw), _ptr(dH), dH.stride(0), _stream()))


def sdt_gat_workspace_bytes(cap_src: int, cap_dst: int, F: int) -> int:
    return lib().sdt_gat_workspace_bytes(cap_src, cap_dst, F)


def sdt_gat_aggregate_fwd(blk: Block, z: torch.Tensor, a_src: torch.Tensor, a_dst: torch.Tensor, slope: float,
                          out: torch.Tensor, ws: torch.Tensor):
    assert out.dtype == z.dtype
    _check(lib().sdt_gat_aggregate_fwd(ctypes.byref(blk.c), _ptr(z), z.stride(0), z.shape[1], dtype_code(z), _ptr(a_src),
                                       _ptr(a_dst), slope, _ptr(out), out.stride(0), _ptr(ws),
                                       ws.numel() * ws.element_size(), _stream()))


def sdt_gat_aggregate_bwd(blk: Block, z: torch.Tensor, a_src: torch.Tensor, a_dst: torch.Tensor, slope: float,
                          g: torch.Tensor, dz: torch.Tensor, da_src: torch.Tensor, da_dst: torch.Tensor,
                          ws: torch.Tensor):
    assert g.dtype == z.dtype and dz.dtype == z.dtype
    _check(lib().sdt_gat_aggregate_bwd(ctypes.byref(blk.c), _ptr(z), z.stride(0), z.shape[1], dtype_code(z), _ptr(a_src),
                                       _ptr(a_dst), slope, _ptr(g), g.stride(0), _ptr(dz), dz.stride(0), _ptr(da_src),
                                       _ptr(da_dst), _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def sdt_infer_layerwise_workspace_bytes(n_nodes: int, model: sdt_model, dtype: int) -> int:
    return lib().sdt_infer_layerwise_workspace_bytes(n_nodes, ctypes.byref(model), dtype)


def sdt_infer_layerwise(graph: Csr, X: torch.Tensor, model: sdt_model, logits: torch.Tensor, ws: torch.Tensor):
    """logits: fp32 [n_nodes, dims[L]] on the device."""
    assert logits.dtype == torch.float32 and logits.stride(1) == 1
    _check(lib().sdt_infer_layerwise(ctypes.byref(graph.c), _ptr(X), X.stride(0), dtype_code(X), ctypes.byref(model),
                                     _ptr(logits), logits.stride(0), _ptr(ws), ws.numel() * ws.element_size(),
                                     _stream()))


def sdt_model_average(params: Sequence[torch.Tensor], alpha: Sequence[float], out: torch.Tensor):
    """out = sum_i alpha[i] * params[i] (fp32 tensors of one size; out may be one of them)."""
    n = out.numel()
    assert all(p.dtype == torch.float32 and p.is_contiguous() and p.numel() == n for p in params)
    assert out.dtype == torch.float32 and out.is_contiguous() and len(alpha) == len(params)
    ptrs = (_vp * len(params))(*[p.data_ptr() for p in params])
    al = (ctypes.c_float * len(alpha))(*alpha)
    _check(lib().sdt_model_average(ptrs, al, len(params), n, _ptr(out), _stream()))


def make_partition(graph: Csr, X: torch.Tensor, labels: torch.Tensor, seeds: torch.Tensor, n_train: int) -> sdt_partition:
    """seeds: int32 [n_steps, batch] on the device."""
    assert seeds.dim() == 2 and seeds.is_contiguous() and seeds.dtype == torch.int32
    p = sdt_partition()
    p.graph = graph.c
    p.X, p.ldx, p.labels, p.seeds = X.data_ptr(), X.stride(0), labels.data_ptr(), seeds.data_ptr()
    p.n_steps, p.reserved, p.n_train = seeds.shape[0], 0, n_train
    return p


def sdt_train_round_workspace_bytes(parts: Sequence[sdt_partition], batch: int, fanouts: Sequence[int],
                                    model: sdt_model, dtype: int) -> int:
    arr = (sdt_partition * len(parts))(*parts)
    f = (_i32 * len(fanouts))(*fanouts)
    return lib().sdt_train_round_workspace_bytes(arr, len(parts), batch, f, ctypes.byref(model), dtype)


def sdt_train_round(parts: Sequence[sdt_partition], dtype: int, batch: int, fanouts: Sequence[int],
                    global_model: sdt_model, local_models: Sequence[sdt_model], seed: int, first_step: int, lr: float,
                    losses: torch.Tensor, ws: torch.Tensor, aux_streams=None):
    arr = (sdt_partition * len(parts))(*parts)
    loc = (sdt_model * len(local_models))(*local_models)
    f = (_i32 * len(fanouts))(*fanouts)
    main = _stream()
    aux, n_aux = _aux_array(aux_streams)
    _check(lib().sdt_train_round(arr, len(parts), dtype, batch, f, ctypes.byref(global_model), loc, seed, first_step,
                                 lr, _ptr(losses), _ptr(ws), ws.numel() * ws.element_size(), main, aux, n_aux))


def sdt_timing_create(max_steps: int, stage_mask: int) -> ctypes.c_void_p:
    h = ctypes.c_void_p()
    _check(lib().sdt_timing_create(max_steps, stage_mask, ctypes.byref(h)))
    return h


def sdt_timing_create_wide(max_steps: int, stage_mask: int) -> ctypes.c_void_p:
    """stage_mask: a Python int of up to 64 * SDT_STAGE_MASK_WORDS bits."""
    words = (_u64 * SDT_STAGE_MASK_WORDS)(*[(stage_mask >> (64 * w)) & ((1 << 64) - 1) for w in range(SDT_STAGE_MASK_WORDS)])
    h = ctypes.c_void_p()
    _check(lib().sdt_timing_create_wide(max_steps, words, ctypes.byref(h)))
    return h


def sdt_timing_destroy(handle):
    lib().sdt_timing_destroy(handle)


def sdt_timing_reset(handle):
    lib().sdt_timing_reset(handle)


def sdt_timing_set_stride(handle, stride: int):
    _check(lib().sdt_timing_set_stride(handle, stride))


def sdt_timing_read(handle, kind: int, layer: int, max_steps: int) -> List[float]:
    buf = (ctypes.c_float * max_steps)()
    n = _i32(0)
    _check(lib().sdt_timing_read(handle, kind, layer, buf, ctypes.byref(n)))
    return list(buf[:n.value])


class Timing:
    """Owner of an sdt_timing object: HIP events around selected (stage, layer) pairs."""

    def __init__(self, max_steps: int, stages: Sequence, stride: int = 1):
        mask = 0
        for kind, layer in stages:
            mask |= 1 << (STAGES[kind] * SDT_MAX_LAYERS + layer)
        self.max_steps = max_steps
        self.handle = sdt_timing_create_wide(max_steps, mask)
        if stride != 1:
            sdt_timing_set_stride(self.handle, stride)

    def reset(self):
        sdt_timing_reset(self.handle)

    def read(self, kind: str, layer: int = 0) -> List[float]:
        """Milliseconds per timed step (waits for the events)."""
        return sdt_timing_read(self.handle, STAGES[kind], layer, self.max_steps)

    def close(self):
        if self.handle:
            sdt_timing_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ----------------------------------------------------------------- workspace views (for inspection)
def ws_view(ws: torch.Tensor, offset: int, shape, dtype: torch.dtype) -> torch.Tensor:
    """A tensor view of `shape`/`dtype` at byte `offset` of the uint8 workspace."""
    n = 1
    for s in shape:
        n *= s
    nbytes = n * torch.empty((), dtype=dtype).element_size()
    return ws[offset:offset + nbytes].view(dtype).view(*shape)
