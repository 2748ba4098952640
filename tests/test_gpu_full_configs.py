"""GPU parity at the full sizes of the five workloads, for the step counts they prescribe.
Sequential sdt_train_step calls: index structures against the oracle on every step, floats on
steps 0, 1 and the last, teacher-forced from the GPU's weights (oracle steps cost seconds each).
Then the launch configuration bench.py times -- one sdt_train_loop call over the same
mini-batches, sampling on two auxiliary streams -- must reproduce every loss and the final
weights bit for bit (Sec. III-D: a worker trains many mini-batches between two
synchronisations; that loop is the unit that matters)."""
import functools
import time

import numpy as np
import pytest
import torch

import sdt_gen as gen
from oracle import sdt_oracle as orc
from paper_2404_02300_amd import binding as B
from parity_util import TOL, assert_close, bf16_from_bits, dev, f64, gat_relu_window, relu_window
from test_gpu_parity import _loop_against_steps, _run_and_check, _say

pytestmark = pytest.mark.gpu


@functools.lru_cache(maxsize=1)
def _instance(name):
    """The workload's graph, features and weights; the tests of one workload follow each other and share it."""
    t = time.time()
    inst = gen.make_instance(gen.WORKLOADS[name])
    _say(f"{name}: generated in {time.time() - t:.1f}s, nnz={inst.indptr[-1]}")
    return inst


@pytest.mark.timeout(600)
def test_products_full_size():
    wl = gen.WORKLOADS["products"]
    inst = _instance("products")
    # 100 steps as the workload prescribes: indices every step, floats at 0, 1 and the last;
    # then the same 100 steps through one sdt_train_loop call, as bench.py times them
    seq, losses = _run_and_check(inst, wl, steps=wl.steps, check_float_steps=(0, 1, wl.steps - 1))
    _loop_against_steps(inst, wl, seq, losses)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("kind", ["gcn", "gat"])
def test_products_full_size_other_model_kinds(kind):
    _other_model_kinds("products", kind, 2)


@pytest.mark.timeout(600)
def test_products_spring_full_size():
    """The step on partition 0 of 4 of the products-shaped graph as the streaming partitioner cuts it
    (owned nodes + replicas; the workload of `bench.py --workload products_spring`)."""
    wl = gen.WORKLOADS["products"]
    t = time.time()
    inst = gen.make_partition_instance(wl, p=4, which=0)
    _say(f"products_spring: generated in {time.time() - t:.1f}s, {inst.info}")
    assert inst.n_owned < inst.n_nodes
    seq, losses = _run_and_check(inst, wl, steps=20, check_float_steps=(0, 19))
    _loop_against_steps(inst, wl, seq, losses)


@pytest.mark.timeout(900)
def test_dense_full_size():
    wl = gen.WORKLOADS["dense"]
    t = time.time()
    inst = gen.make_instance(wl)
    _say(f"dense: generated in {time.time() - t:.1f}s, nnz={inst.indptr[-1]}, "
         f"max degree {np.diff(inst.indptr).max()}")
    assert wl.steps == 100
    seq, losses = _run_and_check(inst, wl, steps=wl.steps, check_float_steps=(0, 1, wl.steps - 1))
    _loop_against_steps(inst, wl, seq, losses)


@pytest.mark.timeout(1500)
def test_sparse_bf16_full_size():
    wl = gen.WORKLOADS["sparse_bf16"]
    inst = _instance("sparse_bf16")
    assert wl.steps == 200
    seq, losses = _run_and_check(inst, wl, steps=wl.steps, check_float_steps=(0, 1, wl.steps - 1))
    _loop_against_steps(inst, wl, seq, losses)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("kind", ["gcn", "gat"])
def test_sparse_bf16_full_size_other_model_kinds(kind):
    _other_model_kinds("sparse_bf16", kind, 1)


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
    # the same layer in one launch (aggregated rows kept in LDS): bit-equal on every row
    Y1 = torch.full((N, O), float("nan"), dtype=torch.float32, device="cuda")
    B.sdt_sage_layer_csr_fwd(g, Xd, dev(W[0]), dev(b[0]), True, Y1)
    torch.cuda.synchronize()
    assert_close(f64(Y1[rt]), refY, TOL[torch.float32], "Y of the one-launch layer (sampled rows)")
    assert torch.equal(Y1, Y), "one-launch layer against the two launches"
    _say(f"fullgraph: one-launch layer bit-equal on all {N} rows; {int((deg > 2048).sum())} rows longer than 2048 edges")


def _other_model_kinds(name, kind, steps):
    """The GCN and GAT kinds of the step at the products-shaped sizes (fp32) and at the sizes of the bf16 workload
    (three layers, bf16 storage; one weight matrix per layer, Glorot-uniform from a seed): loss, activations, every
    gradient and the updated parameters, teacher-forced from the GPU's parameters."""
    wl = gen.WORKLOADS[name]
    inst = _instance(name)
    d, L = wl.dims, len(wl.fanouts)
    bf16 = wl.bf16
    dt = torch.bfloat16 if bf16 else torch.float32
    rng = np.random.default_rng(wl.seed + 100)
    W = [(rng.uniform(-1, 1, size=(d[l], d[l + 1])) * np.sqrt(6.0 / (d[l] + d[l + 1]))).astype(np.float32) for l in range(L)]
    att = [(rng.uniform(-1, 1, size=2 * d[l + 1]) * np.sqrt(6.0 / (d[l + 1] + 1))).astype(np.float32) for l in range(L)]
    g = B.Csr(dev(inst.indptr), dev(inst.indices))
    X, y = (bf16_from_bits(inst.X).cuda() if bf16 else dev(inst.X)), dev(inst.y)
    Wd, bd, ad = [dev(w) for w in W], [dev(v) for v in inst.b], [dev(v) for v in att]
    if kind == "gat":
        model = B.make_model(d, Wd, bd, kind=B.SDT_MODEL_GAT, att=ad, gat_slope=0.2)
    else:
        model = B.make_model(d, Wd, bd, kind=B.SDT_MODEL_GCN)
    lay = B.sdt_train_step_layout(g.n_nodes, wl.batch, wl.fanouts, model, B.SDT_BF16 if bf16 else B.SDT_F32)
    ws = torch.zeros(int(lay.total_bytes), dtype=torch.uint8, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    lr, tol = 0.01, TOL[dt]

    def view(off, cap_rows, rows, cols, dtype=torch.float32):
        return f64(B.ws_view(ws, off, (cap_rows, cols), dtype)[:rows])

    for step in range(steps):
        seeds = inst.batch(step)
        W0, b0, a0 = [f64(w) for w in Wd], [f64(v) for v in bd], [f64(v) for v in ad]
        B.sdt_train_step(g, X, y, dev(seeds.astype(np.int32)), wl.fanouts, model, wl.seed, step, lr, loss, ws)
        torch.cuda.synchronize()

        def oracle(blocks=None, masks=None):
            if kind == "gat":
                return orc.gat_train_step(inst.indptr, inst.indices, inst.X, inst.y, seeds, wl.fanouts, W0, b0, a0, wl.seed,
                                          step, lr, 0.2, blocks=blocks, relu_masks=masks, bf16=bf16)
            return orc.gcn_train_step(inst.indptr, inst.indices, inst.X, inst.y, seeds, wl.fanouts, W0, b0, wl.seed, step, lr,
                                      blocks=blocks, relu_masks=masks, bf16=bf16)

        ref = oracle()
        blocks = ref["blocks"]
        # ReLU decisions within rounding of zero may differ between the two sides: adopt the GPU's after checking that
        # every differing element lies inside the bound the stored operands and the fp32 evaluation imply
        masks, n_diff = [None] * L, 0
        for l in range(L - 1):
            Hg = view(lay.H[l + 1], lay.cap_dst[l], blocks[l].n_dst, d[l + 1], dt)
            masks[l] = Hg > 0
            diff = masks[l] != (ref["H"][l + 1] > 0)
            if not diff.any():
                continue
            n_diff += int(diff.sum())
            F = d[l + 1]
            if kind == "gat":
                attend = lambda z: orc.gat_aggregate_fwd(blocks[l].indptr, blocks[l].cols, z, a0[l][:F], a0[l][F:], 0.2)[0]
                win = gat_relu_window(attend, blocks[l], view(lay.z[l], lay.cap_src[l], blocks[l].n_src, F, dt), ref["Z"][l],
                                      a0[l], b0[l])
            else:
                win = relu_window(view(lay.A[l], lay.cap_dst[l], blocks[l].n_dst, d[l], dt), ref["A"][l],
                                  orc.round_bf16(W0[l]) if bf16 else W0[l], b0[l])
            win = win * (1.0 + (2.0 ** -8 if bf16 else 0.0))
            mag = np.maximum(np.abs(Hg), np.abs(ref["H"][l + 1]))
            assert not (diff & (mag > win)).any(), f"ReLU decisions of layer {l} differ beyond the rounding window"
        if n_diff:
            ref = oracle(blocks, masks)
        for l in range(L):
            cnt = B.ws_view(ws, lay.counts[l], (4,), torch.int32).cpu().tolist()
            assert cnt[:3] == [blocks[l].n_dst, blocks[l].n_src, blocks[l].nnz]
            cols = B.ws_view(ws, lay.cols[l], (max(lay.cap_nnz[l], 1),), torch.int32)[:blocks[l].nnz].cpu().numpy()
            assert np.array_equal(cols, blocks[l].cols)
            assert_close(view(lay.H[l + 1], lay.cap_dst[l], blocks[l].n_dst, d[l + 1], dt if l < L - 1 else torch.float32),
                         ref["H"][l + 1], tol, f"H[{l + 1}]")
            assert_close(view(lay.dW[l], d[l], d[l], d[l + 1]), ref["dW"][l], tol, f"dW[{l}]")
            assert_close(view(lay.db[l], 1, 1, d[l + 1])[0], ref["db"][l], tol, f"db[{l}]")
            assert_close(f64(Wd[l]), ref["W_new"][l], tol, f"updated W[{l}]")
            assert_close(f64(bd[l]), ref["b_new"][l], tol, f"updated b[{l}]")
            if kind == "gat":
                assert_close(view(lay.z[l], lay.cap_src[l], blocks[l].n_src, d[l + 1], dt), ref["Z"][l], tol, f"z[{l}]")
                assert_close(view(lay.dz[l], lay.cap_src[l], blocks[l].n_src, d[l + 1], dt), ref["dz"][l], tol, f"dz[{l}]")
                assert_close(view(lay.datt[l], 1, 1, 2 * d[l + 1])[0], ref["datt"][l], tol, f"datt[{l}]")
                assert_close(f64(ad[l]), ref["att_new"][l], tol, f"updated att[{l}]")
            else:
                assert_close(view(lay.A[l], lay.cap_dst[l], blocks[l].n_dst, d[l], dt), ref["A"][l], tol, f"A[{l}]")
        assert abs(float(loss) - ref["loss"]) <= tol * max(1.0, abs(ref["loss"]))
        _say(f"  {kind} {name} step {step}: loss {float(loss):.6f} ok ({n_diff} borderline ReLU decisions adopted)")
