"""GPU parity at the full sizes of the five workloads, in the launch configuration
bench.py times.  Index structures are compared on every step; floats on selected
steps, teacher-forced from the GPU's weights (oracle steps cost seconds each)."""
import time

import numpy as np
import pytest
import torch

import sdt_gen as gen
from oracle import sdt_oracle as orc
from paper_2404_02300_amd import binding as B
from parity_util import TOL, assert_close, dev, f64
from test_gpu_parity import _run_and_check, _say

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(600)
def test_products_full_size():
    wl = gen.WORKLOADS["products"]
    t = time.time()
    inst = gen.make_instance(wl)
    _say(f"products: generated in {time.time() - t:.1f}s, nnz={inst.indptr[-1]}")
    # 100 steps as the workload prescribes: indices every step, floats at 0, 1 and the last
    _run_and_check(inst, wl, steps=wl.steps, check_float_steps=(0, 1, wl.steps - 1))


@pytest.mark.timeout(900)
def test_dense_full_size():
    wl = gen.WORKLOADS["dense"]
    t = time.time()
    inst = gen.make_instance(wl)
    _say(f"dense: generated in {time.time() - t:.1f}s, nnz={inst.indptr[-1]}, "
         f"max degree {np.diff(inst.indptr).max()}")
    _run_and_check(inst, wl, steps=12, check_float_steps=(0, 11))


@pytest.mark.timeout(1500)
def test_sparse_bf16_full_size():
    wl = gen.WORKLOADS["sparse_bf16"]
    t = time.time()
    inst = gen.make_instance(wl)
    _say(f"sparse_bf16: generated in {time.time() - t:.1f}s, nnz={inst.indptr[-1]}")
    _run_and_check(inst, wl, steps=12, check_float_steps=(0, 11))


@pytest.mark.timeout(900)
def test_fullgraph_layer_sampled_rows():
    """Full-neighbour layer over all 2^22 nodes: SpMM over the whole CSR, then the projection.
    The oracle recomputes a seeded sample of 2^15 rows plus every maximum-degree row and a
    batch of isolated rows (rows are independent of each other)."""
    wl = gen.WORKLOADS["fullgraph"]
    t = time.time()
    indptr, indices = gen.make_graph(wl)
    X = gen.normal_features(wl.n_nodes, wl.feat, wl.seed)
    W, b = gen.glorot_sage_weights(wl.dims, wl.seed)
    _say(f"fullgraph: generated in {time.time() - t:.1f}s, nnz={indptr[-1]}")
    N, F, O = wl.n_nodes, wl.dims[0], wl.dims[1]
    g = B.Csr(dev(indptr), dev(indices))
    Xd = dev(X)
    A = torch.empty(N, F, dtype=torch.float32, device="cuda")
    Y = torch.empty(N, O, dtype=torch.float32, device="cuda")
    B.sdt_sage_aggregate_csr_fwd(g, Xd, A)
    B.sdt_sage_linear_fwd(Xd, A, dev(W[0]), dev(b[0]), True, Y)
    torch.cuda.synchronize()
    deg = np.diff(indptr)
    rng = np.random.default_rng(wl.seed)
    rows = np.unique(np.concatenate([rng.choice(N, size=1 << 15, replace=False),
                                     np.argsort(deg)[-4:], np.flatnonzero(deg == 0)[:64]]))
    sub_ip = np.zeros(len(rows) + 1, dtype=np.int64)
    sub_ip[1:] = np.cumsum(deg[rows])
    sub_cols = np.concatenate([indices[indptr[r]:indptr[r + 1]] for r in rows]).astype(np.int32)
    refA = orc.aggregate_fwd(sub_ip, sub_cols, X.astype(np.float64))
    rt = torch.from_numpy(rows).cuda()
    assert_close(f64(A[rt]), refA, TOL[torch.float32], "A (sampled rows)")
    iso = deg[rows] == 0
    assert iso.any() and not f64(A[rt])[iso].any()
    refY = orc.linear_fwd(X[rows].astype(np.float64), refA, W[0], b[0], relu=True)
    assert_close(f64(Y[rt]), refY, TOL[torch.float32], "Y (sampled rows)")
    _say(f"fullgraph: {len(rows)} rows checked, max degree {deg.max()}")
