"""GPU parity of the GCN aggregation kernels and of a GCN mini-batch step against the CPU oracle
(fp32: 1e-5 max-norm relative, bf16 storage: 2e-2; index structures bit-exact)."""
import numpy as np
import pytest
import torch

import sdt_gen as gen
from oracle import sdt_oracle as orc
from paper_2404_02300_amd import binding as B
from parity_util import assert_close, bf16_from_bits, dev, f64, gat_relu_window, relu_window, upload_block

pytestmark = pytest.mark.gpu
TOL = 1e-5
TOL_BF16 = 2e-2


def _say(msg):
    print(msg, flush=True)


def _graph(rng, n, avg):
    rows = [np.sort(rng.integers(0, n, size=int(rng.integers(0, 2 * avg + 1)))).astype(np.int32) for _ in range(n)]
    rows[5] = np.sort(rng.integers(0, n, size=700)).astype(np.int32)     # a hub with repeated entries
    indptr = np.zeros(n + 1, dtype=np.int64)
    indptr[1:] = np.cumsum([len(r) for r in rows])
    return indptr, np.concatenate(rows).astype(np.int32)


@pytest.mark.parametrize("F,bf16", [(64, False), (100, False), (602, False), (33, False), (64, True), (602, True), (33, True)])
def test_gcn_kernels(F, bf16):
    _say(f"GCN norm / aggregate fwd / bwd, F={F}, bf16={bf16}")
    rng = np.random.default_rng(F)
    dt = torch.bfloat16 if bf16 else torch.float32
    tol = TOL_BF16 if bf16 else TOL
    n = 3000
    indptr, indices = _graph(rng, n, 10)
    dst = np.concatenate([[5], rng.choice(np.arange(6, n), size=799, replace=False)]).astype(np.int32)
    blk = orc.sample_block(indptr, indices, dst, 8, 17, 3, 1)
    s, c, selfw = orc.gcn_weights(indptr, blk.src_nodes, blk.indptr)
    g = B.Csr(dev(indptr), dev(indices))
    gb = upload_block(blk)
    dc = torch.empty(blk.n_src, dtype=torch.float32, device="cuda")
    ds = torch.empty(blk.n_dst, dtype=torch.float32, device="cuda")
    dself = torch.empty(blk.n_dst, dtype=torch.float32, device="cuda")
    B.sdt_gcn_norm(g, gb, dc, ds, dself)
    assert_close(f64(dc), c, 1e-6, "c")
    assert_close(f64(ds), s, 1e-6, "s")
    assert_close(f64(dself), selfw, 1e-6, "selfw")
    # forward from local rows and straight out of the feature matrix through src_nodes; the oracle gets the
    # stored (rounded) inputs and its own normalisation vectors, the output rounding is inside the tolerance
    Xd = dev(rng.standard_normal((n, F)).astype(np.float32)).to(dt)
    X = f64(Xd)
    Hloc = X[blk.src_nodes]
    ref = orc.gcn_aggregate_fwd(blk.indptr, blk.cols, Hloc, s, c, selfw)
    A = torch.zeros(blk.n_dst, F, dtype=dt, device="cuda")
    B.sdt_gcn_aggregate_fwd(gb, Xd[torch.from_numpy(blk.src_nodes.astype(np.int64)).cuda()].contiguous(), dc, ds, dself, A)
    assert_close(f64(A), ref, tol, "A from local rows")
    A2 = torch.zeros_like(A)
    B.sdt_gcn_aggregate_fwd(gb, Xd, dc, ds, dself, A2, through_src_nodes=True)
    assert torch.equal(A, A2)
    # backward, with and without a ReLU mask
    dAd = dev(rng.standard_normal((blk.n_dst, F)).astype(np.float32)).to(dt)
    refb = orc.gcn_aggregate_bwd(blk.indptr, blk.cols, blk.n_src, f64(dAd), s, c, selfw)
    dH = torch.zeros(blk.n_src, F, dtype=dt, device="cuda")
    B.sdt_gcn_aggregate_bwd(gb, dAd, dc, ds, dself, dH)
    assert_close(f64(dH), refb, tol, "dH")
    Yd = dev(rng.standard_normal((blk.n_src, F)).astype(np.float32)).to(dt)
    B.sdt_gcn_aggregate_bwd(gb, dAd, dc, ds, dself, dH, relu_of=Yd)
    assert_close(f64(dH), refb * (f64(Yd) > 0), tol, "dH masked")


def _view(ws, off, rows_cap, rows, cols, dtype=torch.float32):
    return f64(B.ws_view(ws, off, (rows_cap, cols), dtype)[:rows])


@pytest.mark.parametrize("classes,bf16", [(8, False), (300, False), (8, True), (300, True)])
def test_gcn_train_step(classes, bf16):
    _say(f"GCN train step, {classes} classes, bf16={bf16}")
    wl = gen.Workload("gcn", "rmat", 13, 12, 64, classes, 64, 2, [8, 5], 128, 41, 1, owned_frac=0.5, bf16=bf16)
    inst = gen.make_instance(wl)
    rng = np.random.default_rng(1)
    d = wl.dims
    dt = torch.bfloat16 if bf16 else torch.float32
    tol = TOL_BF16 if bf16 else TOL
    W = [(rng.standard_normal((d[l], d[l + 1])) * (1.0 / np.sqrt(d[l]))).astype(np.float32) for l in range(2)]
    b = [(rng.standard_normal(d[l + 1]) * 0.05).astype(np.float32) for l in range(2)]
    g = B.Csr(dev(inst.indptr), dev(inst.indices))
    X, y = (bf16_from_bits(inst.X).cuda() if bf16 else dev(inst.X)), dev(inst.y)
    Wd, bd = [dev(w) for w in W], [dev(v) for v in b]
    model = B.make_model(d, Wd, bd, kind=B.SDT_MODEL_GCN)
    code = B.SDT_BF16 if bf16 else B.SDT_F32
    lay = B.sdt_train_step_layout(g.n_nodes, wl.batch, wl.fanouts, model, code)
    ws = torch.zeros(int(lay.total_bytes), dtype=torch.uint8, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    lr = 0.05
    for step in range(2):
        seeds = inst.batch(step)
        W0, b0 = [f64(w) for w in Wd], [f64(v) for v in bd]
        B.sdt_train_step(g, X, y, dev(seeds.astype(np.int32)), wl.fanouts, model, wl.seed, step, lr, loss, ws)
        torch.cuda.synchronize()
        ref = orc.gcn_train_step(inst.indptr, inst.indices, inst.X, inst.y, seeds, wl.fanouts, W0, b0, wl.seed, step, lr, bf16=bf16)
        blocks = ref["blocks"]
        # ReLU decisions within rounding of zero may differ between the two sides: adopt the GPU's after checking that
        # every differing element lies inside the bound the operands and the fp32 accumulation imply
        H1 = _view(ws, lay.H[1], lay.cap_dst[0], blocks[0].n_dst, d[1], dt)
        diff = (H1 > 0) != (ref["H"][1] > 0)
        if diff.any():
            A0 = _view(ws, lay.A[0], lay.cap_dst[0], blocks[0].n_dst, d[0], dt)
            w0 = orc.round_bf16(ref["W"][0]) if bf16 else ref["W"][0]
            win = relu_window(A0, ref["A"][0], w0, b0[0]) * (1.0 + (2.0 ** -8 if bf16 else 0.0))
            mag = np.maximum(np.abs(H1), np.abs(ref["H"][1]))
            assert not (diff & (mag > win)).any(), "ReLU decisions differ beyond the rounding window"
            ref = orc.gcn_train_step(inst.indptr, inst.indices, inst.X, inst.y, seeds, wl.fanouts, W0, b0, wl.seed, step, lr,
                                     blocks=blocks, relu_masks=[H1 > 0, None], bf16=bf16)
        for l in range(2):
            cnt = B.ws_view(ws, lay.counts[l], (4,), torch.int32).cpu().tolist()
            assert cnt[:3] == [blocks[l].n_dst, blocks[l].n_src, blocks[l].nnz]
            cols = B.ws_view(ws, lay.cols[l], (max(lay.cap_nnz[l], 1),), torch.int32)[:blocks[l].nnz].cpu().numpy()
            assert np.array_equal(cols, blocks[l].cols)
            assert_close(_view(ws, lay.A[l], lay.cap_dst[l], blocks[l].n_dst, d[l], dt), ref["A"][l], tol, f"A[{l}]")
            assert_close(_view(ws, lay.H[l + 1], lay.cap_dst[l], blocks[l].n_dst, d[l + 1], dt if l == 0 else torch.float32),
                         ref["H"][l + 1], tol, f"H[{l + 1}]")
            assert_close(_view(ws, lay.dW[l], d[l], d[l], d[l + 1]), ref["dW"][l], tol, f"dW[{l}]")
            assert_close(_view(ws, lay.db[l], 1, 1, d[l + 1])[0], ref["db"][l], tol, f"db[{l}]")
            assert_close(f64(Wd[l]), ref["W_new"][l], tol, f"updated W[{l}]")
            assert_close(f64(bd[l]), ref["b_new"][l], tol, f"updated b[{l}]")
        assert_close(_view(ws, lay.dAgg[1], lay.cap_dst[1], blocks[1].n_dst, d[1], dt), ref["dA"][1], tol, "dA[1]")
        assert_close(_view(ws, lay.dH[1], lay.cap_src[1], blocks[1].n_src, d[1], dt),
                     ref["dH"][1] * (ref["H"][1] > 0 if not diff.any() else H1 > 0), tol, "dH[1]")
        assert abs(float(loss) - ref["loss"]) <= tol * max(1.0, abs(ref["loss"]))
        # the next step must not depend on what this one left in the frontier state: poison it
        ws[lay.header:lay.counts[0]].fill_(0x5A)
        _say(f"  step {step}: loss {float(loss):.6f} ok")


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("F,fanout", [(64, 8), (100, 5), (256, 10), (7, 64), (300, 6)])
def test_gat_attention_aggregation(F, fanout, bf16):
    _say(f"GAT attention aggregation fwd / bwd, F={F}, fanout={fanout}, bf16={bf16}")
    rng = np.random.default_rng(F + fanout)
    n = 3000
    indptr, indices = _graph(rng, n, 10)
    dst = np.concatenate([[5], rng.choice(np.arange(6, n), size=599, replace=False)]).astype(np.int32)
    blk = orc.sample_block(indptr, indices, dst, fanout, 23, 1, 0)
    dt = torch.bfloat16 if bf16 else torch.float32
    # bf16 storage: both sides start from the same bf16 numbers; what the kernels store (out, dz) is one rounding away
    # from the fp32 result (2^-9 relative, and the bar is taken at twice that), the fp32 outputs keep the fp32 bar
    tol_stored = 2.0 ** -8 if bf16 else TOL
    zt = torch.from_numpy((rng.standard_normal((blk.n_src, F)) * 0.7).astype(np.float32)).to(dt)
    gt = torch.from_numpy(rng.standard_normal((blk.n_dst, F)).astype(np.float32)).to(dt)
    z, g = f64(zt), f64(gt)
    a_src = (rng.standard_normal(F) * 0.5).astype(np.float32)
    a_dst = (rng.standard_normal(F) * 0.5).astype(np.float32)
    ref, _, _ = orc.gat_aggregate_fwd(blk.indptr, blk.cols, z, a_src, a_dst, 0.2)
    rdz, rda_s, rda_d = orc.gat_aggregate_bwd(blk.indptr, blk.cols, z, a_src, a_dst, g, 0.2)
    gb = upload_block(blk)
    ws = torch.empty(B.sdt_gat_workspace_bytes(blk.n_src, blk.n_dst, F), dtype=torch.uint8, device="cuda")
    dzz, dg, das, dad = zt.cuda(), gt.cuda(), dev(a_src), dev(a_dst)
    out = torch.full((blk.n_dst, F), float("nan"), dtype=dt, device="cuda")
    B.sdt_gat_aggregate_fwd(gb, dzz, das, dad, 0.2, out, ws)
    assert_close(f64(out), ref, tol_stored, "attention output")
    dz = torch.full((blk.n_src, F), float("nan"), dtype=dt, device="cuda")
    da_s = torch.zeros(F, dtype=torch.float32, device="cuda")
    da_d = torch.zeros(F, dtype=torch.float32, device="cuda")
    B.sdt_gat_aggregate_bwd(gb, dzz, das, dad, 0.2, dg, dz, da_s, da_d, ws)
    assert_close(f64(dz), rdz, tol_stored, "dz")
    assert_close(f64(da_s), rda_s, TOL, "da_src")
    assert_close(f64(da_d), rda_d, TOL, "da_dst")
    # deterministic: a second run gives the same bits
    dz2 = torch.empty_like(dz)
    B.sdt_gat_aggregate_fwd(gb, dzz, das, dad, 0.2, out, ws)
    B.sdt_gat_aggregate_bwd(gb, dzz, das, dad, 0.2, dg, dz2, da_s, da_d, ws)
    assert torch.equal(dz, dz2)
    with pytest.raises(B.SdtError) as e:
        B.sdt_gat_aggregate_fwd(gb, dzz, das, dad, 0.2, out, ws[:64])
    assert e.value.code == B.SDT_ERR_WORKSPACE


def _gat_setup(classes, seed, bf16=False, hidden=64):
    wl = gen.Workload("gat", "rmat", 13, 12, 64, classes, hidden, 2, [8, 5], 128, 43, 1, owned_frac=0.5, bf16=bf16)
    inst = gen.make_instance(wl)
    rng = np.random.default_rng(seed)
    d = wl.dims
    W = [(rng.standard_normal((d[l], d[l + 1])) * (1.0 / np.sqrt(d[l]))).astype(np.float32) for l in range(2)]
    b = [(rng.standard_normal(d[l + 1]) * 0.05).astype(np.float32) for l in range(2)]
    att = [(rng.standard_normal(2 * d[l + 1]) * 0.3).astype(np.float32) for l in range(2)]
    return wl, inst, W, b, att


@pytest.mark.parametrize("classes,adam,bf16,hidden", [
    (8, False, False, 64), (300, False, False, 64), (8, True, False, 64),
    (8, False, True, 64), (300, False, True, 64), (8, True, True, 64),
    # a hidden width that is no multiple of four: the one-feature-per-lane kernels on every tensor of the inner layer
    (8, False, False, 66), (8, False, True, 66)])
def test_gat_train_step(classes, adam, bf16, hidden):
    _say(f"GAT train step, {classes} classes, hidden {hidden}, {'Adam' if adam else 'SGD'}, bf16={bf16}")
    wl, inst, W, b, att = _gat_setup(classes, 3, bf16, hidden)
    d = wl.dims
    dt = torch.bfloat16 if bf16 else torch.float32
    tol = TOL_BF16 if bf16 else TOL
    code = B.SDT_BF16 if bf16 else B.SDT_F32
    g = B.Csr(dev(inst.indptr), dev(inst.indices))
    X, y = (bf16_from_bits(inst.X).cuda() if bf16 else dev(inst.X)), dev(inst.y)
    Wd, bd, ad = [dev(w) for w in W], [dev(v) for v in b], [dev(v) for v in att]
    model = B.make_model(d, Wd, bd, kind=B.SDT_MODEL_GAT, att=ad, gat_slope=0.2)
    if adam:
        zeros = lambda ts: [torch.zeros_like(t) for t in ts]
        mom = dict(mW=zeros(Wd), vW=zeros(Wd), mb=zeros(bd), vb=zeros(bd), matt=zeros(ad), vatt=zeros(ad))
        B.use_adam(model, mom["mW"], mom["vW"], mom["mb"], mom["vb"], 0.9, 0.999, 1e-8, mom["matt"], mom["vatt"])
    lay = B.sdt_train_step_layout(g.n_nodes, wl.batch, wl.fanouts, model, code)
    ws = torch.zeros(int(lay.total_bytes), dtype=torch.uint8, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    lr = 0.05
    for step in range(2):
        seeds = inst.batch(step)
        W0, b0, a0 = [f64(w) for w in Wd], [f64(v) for v in bd], [f64(v) for v in ad]
        if adam:
            m0 = {k: [f64(t) for t in v] for k, v in mom.items()}
        B.sdt_train_step(g, X, y, dev(seeds.astype(np.int32)), wl.fanouts, model, wl.seed, step, lr, loss, ws)
        torch.cuda.synchronize()
        ref = orc.gat_train_step(inst.indptr, inst.indices, inst.X, inst.y, seeds, wl.fanouts, W0, b0, a0, wl.seed, step, lr, 0.2,
                                 bf16=bf16)
        blocks = ref["blocks"]
        # ReLU decisions within rounding of zero may differ between the two sides: adopt the GPU's after checking that
        # every differing element lies inside the bound the stored projected rows and the fp32 evaluation imply
        H1 = _view(ws, lay.H[1], lay.cap_dst[0], blocks[0].n_dst, d[1], dt)
        diff = (H1 > 0) != (ref["H"][1] > 0)
        if diff.any():
            attend = lambda z: orc.gat_aggregate_fwd(blocks[0].indptr, blocks[0].cols, z, a0[0][:d[1]], a0[0][d[1]:], 0.2)[0]
            win = gat_relu_window(attend, blocks[0], _view(ws, lay.z[0], lay.cap_src[0], blocks[0].n_src, d[1], dt), ref["Z"][0],
                                  a0[0], b0[0]) * (1.0 + (2.0 ** -8 if bf16 else 0.0))
            mag = np.maximum(np.abs(H1), np.abs(ref["H"][1]))
            assert not (diff & (mag > win)).any(), "ReLU decisions differ beyond the rounding window"
            ref = orc.gat_train_step(inst.indptr, inst.indices, inst.X, inst.y, seeds, wl.fanouts, W0, b0, a0, wl.seed, step, lr,
                                     0.2, blocks=blocks, relu_masks=[H1 > 0, None], bf16=bf16)
        for l in range(2):
            cnt = B.ws_view(ws, lay.counts[l], (4,), torch.int32).cpu().tolist()
            assert cnt[:3] == [blocks[l].n_dst, blocks[l].n_src, blocks[l].nnz]
            cols = B.ws_view(ws, lay.cols[l], (max(lay.cap_nnz[l], 1),), torch.int32)[:blocks[l].nnz].cpu().numpy()
            assert np.array_equal(cols, blocks[l].cols)
            assert_close(_view(ws, lay.z[l], lay.cap_src[l], blocks[l].n_src, d[l + 1], dt), ref["Z"][l], tol, f"z[{l}]")
            assert_close(_view(ws, lay.H[l + 1], lay.cap_dst[l], blocks[l].n_dst, d[l + 1], dt if l == 0 else torch.float32),
                         ref["H"][l + 1], tol, f"H[{l + 1}]")
            assert_close(_view(ws, lay.dz[l], lay.cap_src[l], blocks[l].n_src, d[l + 1], dt), ref["dz"][l], tol, f"dz[{l}]")
            gW = _view(ws, lay.dW[l], d[l], d[l], d[l + 1])
            gb = _view(ws, lay.db[l], 1, 1, d[l + 1])[0]
            ga = _view(ws, lay.datt[l], 1, 1, 2 * d[l + 1])[0]
            assert_close(gW, ref["dW"][l], tol, f"dW[{l}]")
            assert_close(gb, ref["db"][l], tol, f"db[{l}]")
            assert_close(ga, ref["datt"][l], tol, f"datt[{l}]")
            if not adam:
                assert_close(f64(Wd[l]), ref["W_new"][l], tol, f"updated W[{l}]")
                assert_close(f64(bd[l]), ref["b_new"][l], tol, f"updated b[{l}]")
                assert_close(f64(ad[l]), ref["att_new"][l], tol, f"updated att[{l}]")
            else:
                # the Adam update is ill-conditioned in the gradient (g / (|g| + eps)): check it on the GPU's own gradient
                for name, P0, G, mk, vk, Pd in (("W", W0, gW, "mW", "vW", Wd), ("b", b0, gb, "mb", "vb", bd),
                                                 ("att", a0, ga, "matt", "vatt", ad)):
                    # the decay rates cross the ABI as fp32: the oracle takes the values the library was given
                    w1, m1, v1 = orc.adam(P0[l], G, m0[mk][l], m0[vk][l], step + 1, lr, float(np.float32(0.9)),
                                          float(np.float32(0.999)), float(np.float32(1e-8)))
                    assert_close(f64(Pd[l]), w1, tol, f"Adam {name}[{l}]")
                    assert_close(f64(mom[mk][l]), m1, tol, f"Adam m {name}[{l}]")
                    assert_close(f64(mom[vk][l]), v1, tol, f"Adam v {name}[{l}]")
        mask = (ref["H"][1] > 0) if not diff.any() else (H1 > 0)
        assert_close(_view(ws, lay.dH[1], lay.cap_src[1], blocks[1].n_src, d[1], dt), ref["dH"][1] * mask, tol, "dH[1]")
        assert abs(float(loss) - ref["loss"]) <= tol * max(1.0, abs(ref["loss"]))
        ws[lay.header:lay.counts[0]].fill_(0x5A)   # nothing in the frontier state is carried to the next step
        _say(f"  step {step}: loss {float(loss):.6f} ok")


@pytest.mark.parametrize("bf16", [False, True])
def test_gat_train_loop_equals_steps(bf16):
    _say(f"GAT train loop == steps in sequence, bf16={bf16}")
    wl, inst, W, b, att = _gat_setup(8, 5, bf16)
    d = wl.dims
    code = B.SDT_BF16 if bf16 else B.SDT_F32
    g = B.Csr(dev(inst.indptr), dev(inst.indices))
    X, y = (bf16_from_bits(inst.X).cuda() if bf16 else dev(inst.X)), dev(inst.y)
    n_steps = 7
    seeds = dev(np.stack([inst.batch(s) for s in range(n_steps)]).astype(np.int32))
    results = []
    for mode in ("steps", "loop"):
        Wd, bd, ad = [dev(w) for w in W], [dev(v) for v in b], [dev(v) for v in att]
        model = B.make_model(d, Wd, bd, kind=B.SDT_MODEL_GAT, att=ad, gat_slope=0.2)
        losses = torch.zeros(n_steps, dtype=torch.float32, device="cuda")
        if mode == "steps":
            lay = B.sdt_train_step_layout(g.n_nodes, wl.batch, wl.fanouts, model, code)
            ws = torch.zeros(int(lay.total_bytes), dtype=torch.uint8, device="cuda")
            for s in range(n_steps):
                B.sdt_train_step(g, X, y, seeds[s], wl.fanouts, model, wl.seed, s, 0.05, losses[s:s + 1], ws)
        else:
            nbytes = B.sdt_train_loop_workspace_bytes(g.n_nodes, wl.batch, wl.fanouts, model, code)
            ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
            aux = [torch.cuda.Stream() for _ in range(2)]
            B.sdt_train_loop(g, X, y, seeds, wl.fanouts, model, wl.seed, 0, 0.05, losses, ws, aux_streams=aux)
        torch.cuda.synchronize()
        results.append((losses.cpu(), [w.cpu() for w in Wd], [v.cpu() for v in ad]))
    assert torch.equal(results[0][0], results[1][0])
    for a, c in zip(results[0][1] + results[0][2], results[1][1] + results[1][2]):
        assert torch.equal(a, c)
