"""Shared helpers of the GPU parity tests: the error metric and the glue that
runs one training step through the C ABI and collects what it produced."""
from __future__ import annotations

import numpy as np
import torch

from paper_2404_02300_amd import binding as B

TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2}


def max_rel(got, ref) -> float:
    """Max-norm relative error: max|got - ref| / max|ref| (element-wise relative
    error is undefined at the exact zeros ReLU produces)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    scale = np.max(np.abs(ref))
    err = np.max(np.abs(got - ref))
    return float(err / scale) if scale > 0 else float(err)


def floored_rel(got, ref) -> float:
    """Element-wise relative error with the denominator floored at 1e-3 * max|ref| (reported for
    information beside the max-norm figure, which is the one the tolerance applies to)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    scale = np.max(np.abs(ref))
    if scale == 0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-3 * scale)))


def assert_close(got, ref, tol, what="", log=None):
    e = max_rel(got, ref)
    assert e <= tol, f"{what}: max-norm relative error {e:.3e} > {tol:.1e}"
    if log is not None:
        log.append((what, e, floored_rel(got, ref)))


def relu_window(x_gpu, x_ref, W, b) -> np.ndarray:
    """Element-wise bound on |z_gpu - z_oracle| for z = x W + b, given the operand rows each side
    actually used (x_* = [self | mean], [n, K]) and the weights as they enter the product:
        |x_gpu - x_ref| |W|  +  (K + 2) 2^-24 (|x_gpu| |W| + |b|)
    The first term is the exact first-order effect of the operands' difference (summation
    order and storage rounding of the earlier stages, measured, not assumed); the second is
    the worst-case rounding of an fp32 accumulation of K products plus the bias (unit
    roundoff 2^-24 per operation) against the oracle's fp64 sum.  Two pre-activations that
    fall on different sides of zero are therefore both inside this window."""
    x_gpu, x_ref = np.asarray(x_gpu, np.float64), np.asarray(x_ref, np.float64)
    aw = np.abs(np.asarray(W, np.float64))
    K = x_gpu.shape[1]
    return np.abs(x_gpu - x_ref) @ aw + (K + 2) * 2.0 ** -24 * (np.abs(x_gpu) @ aw + np.abs(np.asarray(b, np.float64)))


def gat_relu_window(attend, blk, z_gpu, z_ref, att, b) -> np.ndarray:
    """Element-wise bound on |pre_gpu - pre_oracle| for the GAT layer's pre-activation pre = GATagg(z) + b, given
    the projected rows each side actually stored (z_gpu, z_ref: [n_src, F]) and `attend(z)` = the fp64 attention
    aggregation of the block on given rows (the oracle's, passed in by the test):
        |attend(z_gpu) - attend(z_ref)|  +  rounding of an fp32 evaluation of attend(z_gpu) + b.
    The first term is the whole effect of the operands' difference (storage rounding and summation order of the
    projection), measured.  The second: a score is a sum of 2F products (error <= (2F + 2) u S, u = 2^-24, S = the
    largest sum_f |z_jf| (|a_src,f| + |a_dst,f|)); an attention weight moves relatively by twice the score error plus
    the roundings of exp, sum and divide (<= (deg + 8) u (1 + S)); the weighted sum adds deg + 2 roundings; all of it
    relative to at most max_j |z_jf| (+ |b_f|).  Two pre-activations on different sides of zero are both inside."""
    z_gpu, z_ref = np.asarray(z_gpu, np.float64), np.asarray(z_ref, np.float64)
    att, b = np.asarray(att, np.float64), np.asarray(b, np.float64)
    F = z_gpu.shape[1]
    u = 2.0 ** -24
    S = float(np.max(np.abs(z_gpu) @ (np.abs(att[:F]) + np.abs(att[F:])))) if z_gpu.size else 0.0
    deg = int(np.max(np.diff(np.asarray(blk.indptr)))) + 1 if len(blk.indptr) > 1 else 1
    rel = 2.0 * (2 * F + 2) * u * S + (deg + 8) * u * (1.0 + S) + (deg + 2) * u
    colmax = np.max(np.abs(z_gpu), axis=0) if z_gpu.size else np.zeros(F)
    return np.abs(attend(z_gpu) - attend(z_ref)) + rel * (colmax + np.abs(b))[None, :]


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def dev(a: np.ndarray, dtype=None) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def bf16_from_bits(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16)


def upload_block(blk) -> B.Block:
    """An oracle-built block as device arrays behind a C struct."""
    return B.Block.from_arrays(dev(blk.indptr), dev(blk.cols) if blk.nnz else torch.zeros(1, dtype=torch.int32).cuda(),
                               blk.n_src, dev(blk.src_nodes) if blk.n_src else None, dev(blk.t_indptr),
                               dev(blk.t_rows) if blk.nnz else torch.zeros(1, dtype=torch.int32).cuda())


class StepRunner:
    """Owns the device copies of one workload and runs sdt_train_step on it."""

    def __init__(self, indptr, indices, X, y, W, b, fanouts, batch, bf16=False):
        self.dt = torch.bfloat16 if bf16 else torch.float32
        self.graph = B.Csr(dev(indptr), dev(indices))
        self.X = bf16_from_bits(X).cuda() if bf16 else dev(X)
        self.y = dev(y)
        self.W = [dev(w) for w in W]
        self.b = [dev(v) for v in b]
        self.dims = [W[0].shape[0] // 2] + [w.shape[1] for w in W]
        self.fanouts = list(fanouts)
        self.L = len(fanouts)
        self.batch = batch
        self.model = B.make_model(self.dims, self.W, self.b)
        self.code = B.SDT_BF16 if bf16 else B.SDT_F32
        self.lay = B.sdt_train_step_layout(self.graph.n_nodes, batch, self.fanouts, self.model, self.code)
        self.ws = torch.empty(int(self.lay.total_bytes), dtype=torch.uint8, device="cuda")
        self.ws[:256].zero_()          # the header: "nothing known about the node map" (see sdt_train_step)
        self.loss = torch.zeros(1, dtype=torch.float32, device="cuda")

    def step(self, seeds: np.ndarray, seed: int, step: int, lr: float):
        self.seeds = dev(seeds.astype(np.int32))
        B.sdt_train_step(self.graph, self.X, self.y, self.seeds, self.fanouts, self.model, seed, step, lr, self.loss,
                         self.ws)
        torch.cuda.synchronize()
        return float(self.loss.item())

    # ---- views into the workspace ------------------------------------------------
    def counts(self, l):
        return B.ws_view(self.ws, self.lay.counts[l], (4,), torch.int32).cpu().numpy()

    def block(self, l):
        lay = self.lay
        n_dst, n_src, nnz, _ = self.counts(l)
        out = dict(n_dst=int(n_dst), n_src=int(n_src), nnz=int(nnz))
        out["indptr"] = B.ws_view(self.ws, lay.indptr[l], (lay.cap_dst[l] + 1,), torch.int32)[:n_dst + 1].cpu().numpy()
        out["cols"] = B.ws_view(self.ws, lay.cols[l], (max(lay.cap_nnz[l], 1),), torch.int32)[:nnz].cpu().numpy()
        out["src_nodes"] = B.ws_view(self.ws, lay.src_nodes[l], (max(lay.cap_src[l], 1),), torch.int32)[:n_src].cpu().numpy()
        if l >= 1:
            out["t_indptr"] = B.ws_view(self.ws, lay.t_indptr[l], (lay.cap_src[l] + 1,), torch.int32)[:n_src + 1].cpu().numpy()
            out["t_rows"] = B.ws_view(self.ws, lay.t_rows[l], (max(lay.cap_nnz[l], 1),), torch.int32)[:nnz].cpu().numpy()
        return out

    def mat(self, off, cap_rows, rows, cols, dtype, ld=None):
        return f64(B.ws_view(self.ws, off, (cap_rows, ld or cols), dtype)[:rows, :cols])

    def H(self, l, rows):
        lay = self.lay
        if l == 0:
            return self.mat(lay.H[0], lay.cap_dst[0], rows, self.dims[0], self.dt, ld=int(lay.ld_in))
        dt = torch.float32 if l == self.L else self.dt
        return self.mat(lay.H[l], lay.cap_dst[l - 1], rows, self.dims[l], dt)

    def A(self, l, rows):
        return self.mat(self.lay.A[l], self.lay.cap_dst[l], rows, self.dims[l], self.dt, ld=int(self.lay.ld_in) if l == 0 else None)

    def dZ(self):
        return self.mat(self.lay.dZ, self.batch, self.batch, self.dims[-1], torch.float32)

    def grad(self, name, l, rows=None):
        lay, d = self.lay, self.dims
        if name == "dW":
            return self.mat(lay.dW[l], 2 * d[l], 2 * d[l], d[l + 1], torch.float32)
        if name == "db":
            return self.mat(lay.db[l], 1, 1, d[l + 1], torch.float32)[0]
        if name == "dH":
            return self.mat(lay.dH[l], lay.cap_src[l], rows, d[l], self.dt)
        return self.mat(getattr(lay, name)[l], lay.cap_dst[l], rows, d[l], self.dt)


def check_step_against_oracle(run: StepRunner, ref: dict, tol: float, floats: bool = True):
    """Index structures bit-exact; floats within tol (max-norm relative).  Returns the tensor with
    the largest max-norm error as (name, max-norm relative error, element-wise relative error
    floored at 1e-3 max|ref|), or None when only the index structures were compared."""
    L = run.L
    for l in range(L):
        got, want = run.block(l), ref["blocks"][l]
        assert (got["n_dst"], got["n_src"], got["nnz"]) == (want.n_dst, want.n_src, want.nnz), f"counts of block {l}"
        assert np.array_equal(got["indptr"], want.indptr), f"indptr of block {l}"
        assert np.array_equal(got["src_nodes"], want.src_nodes), f"src_nodes of block {l}"
        assert np.array_equal(got["cols"], want.cols), f"cols of block {l}"
        if l >= 1:
            assert np.array_equal(got["t_indptr"], want.t_indptr), f"t_indptr of block {l}"
            assert np.array_equal(got["t_rows"], want.t_rows), f"t_rows of block {l}"
    if not floats:
        return None
    log = []
    blocks = ref["blocks"]
    n0 = blocks[0].n_dst            # only the destination prefix of the frontier is copied
    assert np.array_equal(run.H(0, n0), ref["H"][0][:n0]), "gathered features are a bit copy"
    for l in range(L):
        assert_close(run.A(l, blocks[l].n_dst), ref["A"][l], tol, f"A[{l}]", log)
        assert_close(run.H(l + 1, blocks[l].n_dst), ref["H"][l + 1], tol, f"H[{l + 1}]", log)
    assert_close(run.dZ(), ref["dZ"], tol, "dZ", log)
    for l in range(L):
        assert_close(run.grad("dW", l), ref["dW"][l], tol, f"dW[{l}]", log)
        assert_close(run.grad("db", l), ref["db"][l], tol, f"db[{l}]", log)
        if l >= 1:
            assert_close(run.grad("dSelf", l, blocks[l].n_dst), ref["dSelf"][l], tol, f"dSelf[{l}]", log)
            assert_close(run.grad("dAgg", l, blocks[l].n_dst), ref["dAgg"][l], tol, f"dAgg[{l}]", log)
            # the ReLU decisions the oracle's backward used (reconciled ones if present)
            masks = ref.get("relu_masks")
            keep = masks[l - 1] if masks is not None and masks[l - 1] is not None else ref["H"][l] > 0
            masked = ref["dH"][l] * keep
            assert_close(run.grad("dH", l, blocks[l].n_src), masked, tol, f"dH[{l}] (ReLU-masked)", log)
    return max(log, key=lambda t: t[1])
