"""Pins for the CPU oracle: every function is checked against something other
than itself -- published known-answer vectors, invariants, brute force,
hand-built graphs, library routines, closed forms and finite differences."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import sdt_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------- Philox
def test_philox_known_answers():
    n = 0
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(x, 16) for x in line.split()]
        assert list(orc.philox4x32_10(v[:4], v[4:6])) == v[6:]
        n += 1
    assert n == 3


# ----------------------------------------------------------------- sampling
def test_sample_positions_invariants():
    for d, k in [(0, 5), (1, 5), (5, 5), (4, 10), (6, 5), (30, 10), (1000, 25), (100000, 64), (7, 0)]:
        for node in range(20):
            pos = orc.sample_positions(d, k, 1234, 3, 1, node)
            assert len(pos) == min(d, max(k, 0))
            assert np.all(np.diff(pos) > 0)                      # distinct and ascending
            if len(pos):
                assert pos[0] >= 0 and pos[-1] < d
            if d <= k:
                assert list(pos) == list(range(d))               # clamp: the whole row


def test_sample_positions_keyed_by_every_argument():
    base = dict(seed=7, step=11, layer=1, node=99)
    ref = orc.sample_positions(5000, 10, **base)
    assert np.array_equal(ref, orc.sample_positions(5000, 10, **base))
    for name, val in [("seed", 8), ("seed", 7 + (1 << 32)), ("step", 12), ("layer", 0), ("node", 98)]:
        other = dict(base)
        other[name] = val
        assert not np.array_equal(ref, orc.sample_positions(5000, 10, **other)), name


def test_sample_subsets_uniform_chi_square():
    # d=4, k=2: the 6 subsets must be equally likely (chi-square, 5 dof;
    # 20.5 is the 0.1 % point, a wrong index or range gives thousands).
    counts = {}
    n = 60000
    for key in range(n):
        s = tuple(orc.sample_positions(4, 2, key, 0, 0, 5))
        counts[s] = counts.get(s, 0) + 1
    assert len(counts) == 6
    chi2 = sum((c - n / 6) ** 2 / (n / 6) for c in counts.values())
    assert chi2 < 20.5, (chi2, counts)


@pytest.mark.parametrize("d,k", [(30, 10), (1000, 25)])
def test_sample_inclusion_frequency(d, k):
    trials = 6000 if d == 30 else 4000
    hits = np.zeros(d)
    for key in range(trials):
        hits[orc.sample_positions(d, k, 99, key, 0, key % 17)] += 1
    p = k / d
    sigma = math.sqrt(trials * p * (1 - p))
    assert np.all(np.abs(hits - trials * p) < 5.5 * sigma)
    assert hits.sum() == trials * k


def test_sample_matches_explicit_fisher_yates():
    # Same rule on a fully materialised array: swap-based Fisher-Yates driven
    # by the same published generator, written independently with numpy ints.
    d, k, seed, step, layer, node = 37, 9, (5 << 32) | 77, 4, 1, 123
    a = list(range(d))
    out = []
    for i in range(k):
        w = orc.philox4x32_10([i >> 2, node, layer, step], [seed & 0xFFFFFFFF, seed >> 32])[i & 3]
        j = i + ((int(w) * (d - i)) >> 32)
        out.append(a[j])
        a[j] = a[i]
    assert sorted(out) == list(orc.sample_positions(d, k, seed, step, layer, node))


def _random_csr(rng, n, avg_deg, allow_dups=False):
    rows = []
    for v in range(n):
        d = int(rng.integers(0, 2 * avg_deg + 1))
        if allow_dups:
            r = np.sort(rng.integers(0, n, size=d))
        else:
            r = np.sort(rng.choice(n, size=min(d, n), replace=False))
        rows.append(r.astype(np.int32))
    indptr = np.zeros(n + 1, dtype=np.int64)
    indptr[1:] = np.cumsum([len(r) for r in rows])
    return indptr, (np.concatenate(rows) if n else np.zeros(0, np.int32)).astype(np.int32)


def _check_block(indptr, indices, dst, fanout, blk):
    n_dst = len(dst)
    assert blk.n_dst == n_dst
    assert np.array_equal(blk.src_nodes[:n_dst], dst)                       # dst prefix
    assert len(np.unique(blk.src_nodes)) == blk.n_src                        # unique
    tail = blk.src_nodes[n_dst:]
    assert np.all(np.diff(tail) > 0)                                         # ascending tail
    assert np.all((blk.cols >= 0) & (blk.cols < blk.n_src))
    if len(tail):
        assert set(range(n_dst, blk.n_src)) <= set(blk.cols.tolist())        # every new node is used
    for i, v in enumerate(dst):
        row = indices[indptr[v]:indptr[v + 1]]
        got = blk.src_nodes[blk.cols[blk.indptr[i]:blk.indptr[i + 1]]]
        assert len(got) == min(len(row), fanout)
        if len(row) <= fanout:
            assert np.array_equal(got, row)
        else:
            # true neighbours, drawn without replacement (compare as multisets of positions)
            rl = row.tolist()
            for g in got:
                assert g in rl
                rl.remove(g)
    # transposed block holds the same edges, rows ascending per segment
    edges = sorted((int(c), i) for i in range(n_dst) for c in blk.cols[blk.indptr[i]:blk.indptr[i + 1]])
    tedges = [(j, int(r)) for j in range(blk.n_src) for r in blk.t_rows[blk.t_indptr[j]:blk.t_indptr[j + 1]]]
    assert edges == tedges
    assert blk.t_indptr[-1] == blk.nnz


@pytest.mark.parametrize("dups", [False, True])
def test_block_invariants(dups):
    rng = np.random.default_rng(5)
    indptr, indices = _random_csr(rng, 300, 8, allow_dups=dups)
    dst = rng.choice(300, size=40, replace=False).astype(np.int32)
    for fanout in (0, 1, 4, 100):
        blk = orc.sample_block(indptr, indices, dst, fanout, 3, 1, 0)
        _check_block(indptr, indices, dst, fanout, blk)


def test_blocks_chain_and_fanout_order():
    rng = np.random.default_rng(6)
    indptr, indices = _random_csr(rng, 500, 12)
    seeds = rng.choice(500, size=16, replace=False).astype(np.int32)
    blocks = orc.sample_blocks(indptr, indices, seeds, [7, 3], 9, 2)
    # the seeds are sampled with the LAST fan-out, the outer frontier with the first
    assert np.array_equal(blocks[1].src_nodes[:16], seeds)
    assert np.array_equal(blocks[0].src_nodes[:blocks[0].n_dst], blocks[1].src_nodes)
    assert np.max(np.diff(blocks[1].indptr)) <= 3 and np.max(np.diff(blocks[0].indptr)) <= 7
    assert np.max(np.diff(blocks[0].indptr)) > 3
    _check_block(indptr, indices, blocks[1].src_nodes, 7, blocks[0])
    # empty seed set
    empty = orc.sample_blocks(indptr, indices, np.zeros(0, np.int32), [7, 3], 9, 2)
    assert empty[0].n_src == 0 and empty[0].nnz == 0


# ----------------------------------------------------------------- gather
def test_gather_is_bit_copy():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((50, 7)).astype(np.float32)
    X[3, 2] = np.nan
    X[4, 1] = -0.0
    idx = rng.integers(0, 50, size=200).astype(np.int32)
    assert np.array_equal(orc.gather_rows(X, idx).view(np.uint32), X[idx].view(np.uint32))
    Xb = rng.integers(0, 65536, size=(50, 5)).astype(np.uint16)
    assert np.array_equal(orc.gather_rows(Xb, idx), Xb[idx])


# ----------------------------------------------------------------- mean aggregation
def _block_from_rows(rows):
    indptr = np.zeros(len(rows) + 1, dtype=np.int32)
    indptr[1:] = np.cumsum([len(r) for r in rows])
    cols = np.array([c for r in rows for c in r], dtype=np.int32)
    return indptr, cols


def test_aggregate_hand_graphs():
    # star: node 0 is the centre, 1..4 the leaves
    X = np.array([[10., 1.], [2., 4.], [4., 8.], [6., 0.], [8., -4.]])
    ip, cols = _block_from_rows([[1, 2, 3, 4], [0], [0], [0], [0]])
    A = orc.aggregate_fwd(ip, cols, X)
    assert np.array_equal(A[0], [5., 2.])
    for leaf in range(1, 5):
        assert np.array_equal(A[leaf], X[0])
    # path 0-1-2-3
    ip, cols = _block_from_rows([[1], [0, 2], [1, 3], [2]])
    A = orc.aggregate_fwd(ip, cols, X[:4])
    assert np.array_equal(A, [[2., 4.], [7., 4.5], [4., 2.], [4., 8.]])
    # isolated row -> zeros; self-loop -> own row takes part; duplicate edge counts twice
    ip, cols = _block_from_rows([[], [1, 2], [0, 0, 1]])
    A = orc.aggregate_fwd(ip, cols, X[:3])
    assert np.array_equal(A[0], [0., 0.])
    assert np.array_equal(A[1], [3., 6.])
    assert np.allclose(A[2], [(10 + 10 + 2) / 3, (1 + 1 + 4) / 3], rtol=0, atol=1e-15)


def test_aggregate_equals_dense_normalised_adjacency():
    rng = np.random.default_rng(2)
    indptr, indices = _random_csr(rng, 60, 5, allow_dups=True)
    X = rng.standard_normal((60, 9))
    adj = np.zeros((60, 60))
    for v in range(60):
        for u in indices[indptr[v]:indptr[v + 1]]:
            adj[v, u] += 1.0
    deg = adj.sum(1, keepdims=True)
    dense = np.divide(adj @ X, deg, out=np.zeros_like(X), where=deg > 0)
    A = orc.aggregate_fwd(indptr, indices, X)
    assert np.allclose(A, dense, rtol=1e-13, atol=1e-13)
    # full fan-out sampling reproduces the same thing through a block
    dst = np.arange(60, dtype=np.int32)
    blk = orc.sample_block(indptr, indices, dst, 1000, 0, 0, 0)
    A2 = orc.aggregate_fwd(blk.indptr, blk.cols, X[blk.src_nodes])
    assert np.allclose(A2, dense, rtol=1e-13, atol=1e-13)
    # constant features stay constant on rows that have neighbours
    Ac = orc.aggregate_fwd(indptr, indices, np.full((60, 3), 2.5))
    assert np.array_equal(Ac[deg[:, 0] > 0], np.full((int((deg > 0).sum()), 3), 2.5))


# ----------------------------------------------------------------- projection
def test_linear_matches_matmul_and_special_cases():
    rng = np.random.default_rng(3)
    n, fin, fout = 13, 5, 4
    H, A = rng.standard_normal((n + 3, fin)), rng.standard_normal((n, fin))
    W, b = rng.standard_normal((2 * fin, fout)), rng.standard_normal(fout)
    ref = np.concatenate([H[:n], A], axis=1) @ W + b
    assert np.allclose(orc.linear_fwd(H, A, W, b, relu=False), ref, rtol=1e-13, atol=1e-13)
    assert np.allclose(orc.linear_fwd(H, A, W, b, relu=True), np.maximum(ref, 0), rtol=1e-13, atol=1e-13)
    assert np.array_equal(orc.linear_fwd(H, A, np.zeros_like(W), b, relu=False), np.tile(b, (n, 1)))
    Wid = np.concatenate([np.eye(fin), np.zeros((fin, fin))])
    assert np.array_equal(orc.linear_fwd(H, A, Wid, np.zeros(fin), relu=False), H[:n])
    Wid2 = np.concatenate([np.zeros((fin, fin)), np.eye(fin)])
    assert np.array_equal(orc.linear_fwd(H, A, Wid2, np.zeros(fin), relu=False), A)


# ----------------------------------------------------------------- loss
@pytest.mark.parametrize("C", [8, 47, 41, 172])
def test_loss_at_zero_logits_is_log_classes(C):
    B = 6
    y = np.arange(B, dtype=np.int32) % C
    loss, dZ = orc.softmax_xent(np.zeros((B, C)), y)
    assert abs(loss - math.log(C)) < 1e-14
    expect = np.full((B, C), 1.0 / C)
    expect[np.arange(B), y] -= 1.0
    assert np.allclose(dZ, expect / B, rtol=0, atol=1e-16)


def test_loss_matches_library_and_is_shift_invariant():
    rng = np.random.default_rng(4)
    Z = rng.standard_normal((9, 11)) * 5
    y = rng.integers(0, 11, size=9).astype(np.int32)
    loss, dZ = orc.softmax_xent(Z, y)
    zt = torch.tensor(Z, requires_grad=True)
    lt = torch.nn.functional.cross_entropy(zt, torch.tensor(y, dtype=torch.long))
    lt.backward()
    assert abs(loss - lt.item()) < 1e-13
    assert np.allclose(dZ, zt.grad.numpy(), rtol=1e-12, atol=1e-15)
    assert np.allclose(dZ.sum(1), 0, atol=1e-16)
    loss2, _ = orc.softmax_xent(Z + 1000.0, y)                      # max-subtraction
    assert abs(loss - loss2) < 1e-9


# ----------------------------------------------------------------- backward
def _tiny_problem(L, seed=0, n=24, F=3, Hd=4, C=3):
    rng = np.random.default_rng(seed)
    indptr, indices = _random_csr(rng, n, 3, allow_dups=True)
    X = rng.standard_normal((n, F)).astype(np.float32)
    y = rng.integers(0, C, size=n).astype(np.int32)
    dims = [F] + [Hd] * (L - 1) + [C]
    W = [rng.standard_normal((2 * dims[l], dims[l + 1])) * 0.7 for l in range(L)]
    b = [rng.standard_normal(dims[l + 1]) * 0.3 for l in range(L)]
    seeds = rng.choice(n, size=6, replace=False).astype(np.int32)
    fanouts = [3, 2, 2][:L]
    return indptr, indices, X, y, seeds, fanouts, W, b


def _loss_only(blocks, H0, W, b, y_seeds):
    H, _ = orc.forward(blocks, H0, W, b)
    return orc.softmax_xent(H[-1], y_seeds)[0], H


@pytest.mark.parametrize("L", [2, 3])
def test_gradients_by_central_differences(L):
    indptr, indices, X, y, seeds, fanouts, W, b = _tiny_problem(L, seed=L)
    out = orc.train_step(indptr, indices, X, y, seeds, fanouts, W, b, seed=1, step=0, lr=0.0)
    blocks, H0 = out["blocks"], out["H"][0]
    # keep the check meaningful: no pre-activation may sit at the ReLU kink
    for l in range(1, L):
        nz = out["H"][l][np.abs(out["H"][l]) > 0]
        assert np.min(np.abs(nz)) > 1e-4
    h = 1e-6
    ys = y[seeds]
    for l in range(L):
        for P, G in ((W, out["dW"]), (b, out["db"])):
            flat = P[l].reshape(-1)
            g = G[l].reshape(-1)
            for idx in range(flat.size):
                keep = flat[idx]
                flat[idx] = keep + h
                lp, _ = _loss_only(blocks, H0, W, b, ys)
                flat[idx] = keep - h
                lm, _ = _loss_only(blocks, H0, W, b, ys)
                flat[idx] = keep
                fd = (lp - lm) / (2 * h)
                assert abs(fd - g[idx]) <= 1e-6 * max(1.0, abs(g[idx])) + 1e-9, (l, idx, fd, g[idx])


@pytest.mark.parametrize("L", [2, 3])
def test_gradients_match_autograd(L):
    # An independent derivation: the same model written with torch CPU ops in
    # fp64 (index_add for the mean) and differentiated by autograd.
    indptr, indices, X, y, seeds, fanouts, W, b = _tiny_problem(L, seed=10 + L, n=40)
    out = orc.train_step(indptr, indices, X, y, seeds, fanouts, W, b, seed=5, step=3, lr=0.0)
    blocks = out["blocks"]
    Wt = [torch.tensor(w, requires_grad=True) for w in W]
    bt = [torch.tensor(v, requires_grad=True) for v in b]
    h = torch.tensor(X[blocks[0].src_nodes].astype(np.float64))
    inter = []
    for l, blk in enumerate(blocks):
        rows = torch.repeat_interleave(torch.arange(blk.n_dst), torch.tensor(np.diff(blk.indptr)).long())
        agg = torch.zeros(blk.n_dst, h.shape[1], dtype=torch.float64)
        agg = agg.index_add(0, rows, h[torch.tensor(blk.cols).long()])
        m = torch.tensor(np.diff(blk.indptr).astype(np.float64)).clamp(min=1).unsqueeze(1)
        z = torch.cat([h[:blk.n_dst], agg / m], dim=1) @ Wt[l] + bt[l]
        h = torch.relu(z) if l < L - 1 else z
        h.retain_grad()
        inter.append(h)
    loss = torch.nn.functional.cross_entropy(h, torch.tensor(y[seeds]).long())
    loss.backward()
    assert abs(loss.item() - out["loss"]) < 1e-12
    for l in range(L):
        assert np.allclose(out["dW"][l], Wt[l].grad.numpy(), rtol=1e-10, atol=1e-13)
        assert np.allclose(out["db"][l], bt[l].grad.numpy(), rtol=1e-10, atol=1e-13)
    for l in range(1, L):
        # dH[l] is the gradient w.r.t. the activations entering layer l
        assert np.allclose(out["dH"][l], inter[l - 1].grad.numpy(), rtol=1e-10, atol=1e-13)


def test_aggregate_bwd_is_the_transpose_of_fwd():
    rng = np.random.default_rng(8)
    indptr, indices = _random_csr(rng, 80, 6, allow_dups=True)
    dst = rng.choice(80, size=20, replace=False).astype(np.int32)
    blk = orc.sample_block(indptr, indices, dst, 4, 2, 0, 1)
    H = rng.standard_normal((blk.n_src, 5))
    G = rng.standard_normal((blk.n_dst, 5))
    S = rng.standard_normal((blk.n_dst, 5))
    A = orc.aggregate_fwd(blk.indptr, blk.cols, H)
    dH = orc.aggregate_bwd(blk.indptr, blk.cols, blk.n_src, G, None)
    assert abs((A * G).sum() - (H * dH).sum()) < 1e-11                      # <A(H),G> = <H,A^T(G)>
    dH2 = orc.aggregate_bwd(blk.indptr, blk.cols, blk.n_src, G, S)
    assert np.allclose(dH2[:blk.n_dst] - dH[:blk.n_dst], S, atol=1e-14)
    has = np.diff(blk.indptr) > 0
    assert np.allclose(dH2.sum(0), S.sum(0) + G[has].sum(0), atol=1e-12)   # conservation
    # the same result through the transposed block (what a gather-style kernel reads)
    m = np.diff(blk.indptr).astype(np.float64)
    viaT = np.zeros_like(dH)
    for j in range(blk.n_src):
        for r in blk.t_rows[blk.t_indptr[j]:blk.t_indptr[j + 1]]:
            viaT[j] += G[r] / m[r]
    assert np.allclose(viaT, dH, atol=1e-14)


# ----------------------------------------------------------------- update
def test_sgd_step():
    indptr, indices, X, y, seeds, fanouts, W, b = _tiny_problem(2, seed=21)
    out0 = orc.train_step(indptr, indices, X, y, seeds, fanouts, W, b, seed=1, step=0, lr=0.0)
    for l in range(2):
        assert np.array_equal(out0["W_new"][l], W[l]) and np.array_equal(out0["b_new"][l], b[l])
    out1 = orc.train_step(indptr, indices, X, y, seeds, fanouts, W, b, seed=1, step=0, lr=0.05)
    assert np.allclose(out1["W_new"][0], W[0] - 0.05 * out0["dW"][0], rtol=0, atol=1e-15)
    out2 = orc.train_step(indptr, indices, X, y, seeds, fanouts, out1["W_new"], out1["b_new"], seed=1, step=0, lr=0.0)
    assert out2["loss"] < out0["loss"]


# ----------------------------------------------------------------- bf16 storage
def test_round_bf16_matches_library_rounding():
    rng = np.random.default_rng(11)
    x32 = np.concatenate([
        rng.standard_normal(5000).astype(np.float32) * np.float32(10.0) ** rng.integers(-30, 30, 5000).astype(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, -3e-39, 65280.0], dtype=np.float32)])
    got = orc.round_bf16(x32.astype(np.float64))
    ref = torch.tensor(x32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, ref)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert orc.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert orc.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    bits = np.array([0x3F80, 0xC000, 0x0001, 0x7F7F], dtype=np.uint16)
    assert np.array_equal(orc.bf16_bits_to_f64(bits), [1.0, -2.0, 2.0 ** -133, 3.3895313892515355e38])


def test_bf16_step_rounds_only_where_stored():
    indptr, indices, X, y, seeds, fanouts, W, b = _tiny_problem(3, seed=33, n=40, F=4, Hd=6, C=5)
    Xb = (torch.tensor(X).to(torch.bfloat16).view(torch.int16).numpy()).view(np.uint16)
    out = orc.train_step(indptr, indices, Xb, y, seeds, fanouts, W, b, seed=2, step=1, lr=0.1, bf16=True)
    is_bf16 = lambda t: np.array_equal(orc.round_bf16(t), t)
    assert all(is_bf16(a) for a in out["A"]) and all(is_bf16(h) for h in out["H"][:-1])
    assert not is_bf16(out["logits"])
    assert all(is_bf16(out["dSelf"][l]) and is_bf16(out["dAgg"][l]) and is_bf16(out["dH"][l]) for l in (1, 2))
    ref = orc.train_step(indptr, indices, orc.bf16_bits_to_f64(Xb).astype(np.float32), y, seeds, fanouts, W, b,
                         seed=2, step=1, lr=0.1)
    assert abs(out["loss"] - ref["loss"]) < 2e-2 * max(1.0, abs(ref["loss"]))
    for l in range(3):
        assert np.max(np.abs(out["dW"][l] - ref["dW"][l])) <= 3e-2 * np.max(np.abs(ref["dW"][l]))


# ----------------------------------------------------------------- layer-wise inference, model averaging
def test_infer_layerwise_equals_dense_matrix_chain():
    # independent formulation: row-normalised dense adjacency, plain matrix products
    rng = np.random.default_rng(11)
    n, dims = 40, [6, 9, 4]
    rows = [np.sort(rng.choice(n, size=int(rng.integers(0, 7)), replace=False)) for _ in range(n)]
    indptr = np.zeros(n + 1, dtype=np.int64)
    indptr[1:] = np.cumsum([len(r) for r in rows])
    indices = np.concatenate(rows).astype(np.int32)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    W = [rng.standard_normal((2 * dims[l], dims[l + 1])) * 0.3 for l in range(2)]
    b = [rng.standard_normal(dims[l + 1]) * 0.1 for l in range(2)]
    P = np.zeros((n, n))
    for v, r in enumerate(rows):
        for u in r:
            P[v, u] += 1.0 / len(r)
    H = X.astype(np.float64)
    for l in range(2):
        Z = H @ W[l][:dims[l]] + (P @ H) @ W[l][dims[l]:] + b[l]
        H = np.maximum(Z, 0) if l == 0 else Z
    got = orc.infer_layerwise(indptr, indices, X, W, b)
    assert np.allclose(got, H, rtol=1e-12, atol=1e-12)
    # an isolated node sees only its own features
    iso = [v for v, r in enumerate(rows) if len(r) == 0]
    assert iso, "the fixture should contain an isolated node"


def test_infer_layerwise_agrees_with_a_full_fanout_training_forward():
    # with fan-outs >= the maximum degree, sampling keeps every neighbour, so the logits of the
    # seeds in a training step equal the layer-wise inference logits of the same nodes
    rng = np.random.default_rng(12)
    n, dims = 60, [5, 7, 3]
    rows = [np.sort(rng.choice(n, size=int(rng.integers(0, 6)), replace=False)) for _ in range(n)]
    indptr = np.zeros(n + 1, dtype=np.int64)
    indptr[1:] = np.cumsum([len(r) for r in rows])
    indices = np.concatenate(rows).astype(np.int32)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    y = rng.integers(0, dims[2], size=n).astype(np.int32)
    W = [rng.standard_normal((2 * dims[l], dims[l + 1])) * 0.3 for l in range(2)]
    b = [rng.standard_normal(dims[l + 1]) * 0.1 for l in range(2)]
    seeds = np.array([3, 17, 42, 0, 59], dtype=np.int32)
    step = orc.train_step(indptr, indices, X, y, seeds, [8, 8], W, b, seed=5, step=0, lr=0.0)
    full = orc.infer_layerwise(indptr, indices, X, W, b)
    assert np.allclose(step["logits"], full[seeds], rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("kind", ["gcn", "gat"])
def test_infer_layerwise_other_kinds(kind):
    """The GCN and GAT passes over the whole graph: (a) against dense formulations written with torch (GCN: the
    symmetric normalised adjacency with self loops; GAT: a dense softmax weighted by edge multiplicities, self edge included), (b) against the
    logits of the seeds in a training step whose fan-outs keep every neighbour."""
    rng = np.random.default_rng(14)
    n, dims = 50, [6, 8, 3]
    rows = [np.sort(rng.choice(n, size=int(rng.integers(0, 6)), replace=False)) for _ in range(n)]
    indptr = np.zeros(n + 1, dtype=np.int64)
    indptr[1:] = np.cumsum([len(r) for r in rows])
    indices = np.concatenate(rows).astype(np.int32)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    y = rng.integers(0, dims[2], size=n).astype(np.int32)
    W = [rng.standard_normal((dims[l], dims[l + 1])) * 0.4 for l in range(2)]
    b = [rng.standard_normal(dims[l + 1]) * 0.1 for l in range(2)]
    att = [rng.standard_normal(2 * dims[l + 1]) * 0.5 for l in range(2)]
    got = orc.infer_layerwise(indptr, indices, X, W, b, kind=kind, att=att)
    Adj = torch.zeros((n, n), dtype=torch.float64)
    for v, r in enumerate(rows):
        for u in r:
            Adj[v, u] += 1.0
    H = torch.tensor(X, dtype=torch.float64)
    for l in range(2):
        if kind == "gcn":
            dinv = torch.diag((Adj.sum(dim=1) + 1.0) ** -0.5)
            Z = dinv @ (Adj + torch.eye(n, dtype=torch.float64)) @ dinv @ H @ torch.tensor(W[l]) + torch.tensor(b[l])
        else:
            F = dims[l + 1]
            z = H @ torch.tensor(W[l])
            score = torch.nn.functional.leaky_relu((z @ torch.tensor(att[l][F:]))[:, None] + (z @ torch.tensor(att[l][:F]))[None, :], 0.2)
            # an edge v -> v in the graph counts beside the built-in self edge: the mask holds multiplicities
            wgt = (Adj + torch.eye(n, dtype=torch.float64)) * torch.exp(score - score.max())
            Z = (wgt / wgt.sum(dim=1, keepdim=True)) @ z + torch.tensor(b[l])
        H = torch.relu(Z) if l == 0 else Z
    assert np.allclose(got, H.numpy(), rtol=1e-11, atol=1e-12)
    assert any(len(r) == 0 for r in rows), "the fixture should contain an isolated node"
    seeds = np.array([3, 17, 42, 0, 49], dtype=np.int32)
    if kind == "gcn":
        step = orc.gcn_train_step(indptr, indices, X, y, seeds, [8, 8], W, b, seed=5, step=0, lr=0.0)
    else:
        step = orc.gat_train_step(indptr, indices, X, y, seeds, [8, 8], W, b, att, seed=5, step=0, lr=0.0)
    assert np.allclose(step["logits"], got[seeds], rtol=1e-11, atol=1e-12)


def test_model_average_closed_forms():
    rng = np.random.default_rng(13)
    a, c = rng.standard_normal(50), rng.standard_normal(50)
    assert np.array_equal(orc.model_average([a, a, a], [5, 1, 9]), a * (5 / 15) + a * (1 / 15) + a * (9 / 15))
    assert np.allclose(orc.model_average([a, a], [3, 4]), a, rtol=1e-15)           # identical models stay put
    assert np.array_equal(orc.model_average([a, c], [7, 0]), a)                     # a worker without training nodes
    assert np.allclose(orc.model_average([a, c], [1, 1]), (a + c) / 2, rtol=1e-15)  # equal shares: plain mean
    got = orc.model_average([np.array([1.0, 2.0]), np.array([5.0, -2.0])], [1, 3])  # worked by hand
    assert np.allclose(got, [4.0, -1.0])
    # the weights sum to one: a constant shift of every model shifts the average by the same constant
    assert np.allclose(orc.model_average([a + 2, c + 2], [2, 5]), orc.model_average([a, c], [2, 5]) + 2)


# ----------------------------------------------------------------- GCN
def _small_graph(rng, n, max_deg):
    rows = [np.sort(rng.choice(n, size=int(rng.integers(0, max_deg + 1)), replace=False)) for _ in range(n)]
    indptr = np.zeros(n + 1, dtype=np.int64)
    indptr[1:] = np.cumsum([len(r) for r in rows])
    return rows, indptr, np.concatenate(rows).astype(np.int32)


def test_gcn_full_fanout_equals_symmetric_normalised_adjacency():
    # every neighbour sampled: the block aggregation is D~^-1/2 (Adj + I) D~^-1/2 H, rows of the seeds
    rng = np.random.default_rng(21)
    n, F = 50, 7
    rows, indptr, indices = _small_graph(rng, n, 6)
    H = rng.standard_normal((n, F))
    Adj = np.zeros((n, n))
    for v, r in enumerate(rows):
        Adj[v, r] = 1.0
    deg = Adj.sum(axis=1)
    Dm = np.diag(1.0 / np.sqrt(deg + 1.0))
    dense = Dm @ (Adj + np.eye(n)) @ Dm @ H          # uses deg(j) of the SOURCE's own row, as gcn_weights does
    dst = np.array([4, 9, 23, 0, 49, 31], dtype=np.int32)
    blk = orc.sample_block(indptr, indices, dst, 8, 3, 0, 0)
    s, c, selfw = orc.gcn_weights(indptr, blk.src_nodes, blk.indptr)
    got = orc.gcn_aggregate_fwd(blk.indptr, blk.cols, H[blk.src_nodes], s, c, selfw)
    assert np.allclose(got, dense[dst], rtol=1e-12, atol=1e-13)
    # sampling fewer neighbours rescales the neighbour sum by deg/m: constant features stay put
    blk2 = orc.sample_block(indptr, indices, dst, 2, 3, 0, 0)
    s2, c2, self2 = orc.gcn_weights(indptr, blk2.src_nodes, blk2.indptr)
    m = np.diff(blk2.indptr)
    assert np.allclose(s2[m > 0] * m[m > 0], deg[dst][m > 0] / np.sqrt(deg[dst][m > 0] + 1))
    assert np.allclose(self2, 1.0 / (deg[dst] + 1))


def test_gcn_aggregate_bwd_is_the_transpose_of_fwd():
    rng = np.random.default_rng(22)
    n, F = 80, 5
    rows, indptr, indices = _small_graph(rng, n, 9)
    dst = rng.choice(n, size=20, replace=False).astype(np.int32)
    blk = orc.sample_block(indptr, indices, dst, 4, 1, 2, 1)
    wt = orc.gcn_weights(indptr, blk.src_nodes, blk.indptr)
    h = rng.standard_normal((blk.n_src, F))
    g = rng.standard_normal((blk.n_dst, F))
    lhs = np.sum(orc.gcn_aggregate_fwd(blk.indptr, blk.cols, h, *wt) * g)
    rhs = np.sum(h * orc.gcn_aggregate_bwd(blk.indptr, blk.cols, blk.n_src, g, *wt))
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))


def test_gcn_step_gradients_match_autograd_on_a_dense_formulation():
    rng = np.random.default_rng(23)
    n, dims = 40, [6, 8, 3]
    rows, indptr, indices = _small_graph(rng, n, 5)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    y = rng.integers(0, dims[2], size=n).astype(np.int32)
    W = [rng.standard_normal((dims[l], dims[l + 1])) * 0.4 for l in range(2)]
    b = [rng.standard_normal(dims[l + 1]) * 0.1 for l in range(2)]
    seeds = np.array([1, 5, 17, 33, 8], dtype=np.int32)
    ref = orc.gcn_train_step(indptr, indices, X, y, seeds, [3, 2], W, b, seed=9, step=4, lr=0.1)
    # the same computation with dense per-block operators and torch autograd in float64
    Wt = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in W]
    bt = [torch.tensor(v, dtype=torch.float64, requires_grad=True) for v in b]
    H = torch.tensor(X[ref["blocks"][0].src_nodes].astype(np.float64))
    for l, blk in enumerate(ref["blocks"]):
        s, c, selfw = ref["weights"][l]
        Pm = np.zeros((blk.n_dst, blk.n_src))
        for i in range(blk.n_dst):
            for e in range(blk.indptr[i], blk.indptr[i + 1]):
                Pm[i, blk.cols[e]] += s[i] * c[blk.cols[e]]
            Pm[i, i] += selfw[i]
        Z = torch.tensor(Pm) @ H @ Wt[l] + bt[l]
        H = torch.relu(Z) if l == 0 else Z
    loss = torch.nn.functional.cross_entropy(H, torch.tensor(y[seeds].astype(np.int64)))
    loss.backward()
    assert abs(loss.item() - ref["loss"]) < 1e-12
    for l in range(2):
        assert np.allclose(ref["dW"][l], Wt[l].grad.numpy(), rtol=1e-10, atol=1e-12)
        assert np.allclose(ref["db"][l], bt[l].grad.numpy(), rtol=1e-10, atol=1e-12)
        assert np.allclose(ref["W_new"][l], W[l] - 0.1 * Wt[l].grad.numpy(), rtol=1e-12, atol=1e-13)


def test_gcn_step_bf16_rounding_points():
    """bf16 storage of the GCN step: the forward equals a float64 computation in which torch's own bf16 cast (an
    independent round-to-nearest-even) is applied to the aggregated rows, the weights and the hidden activations;
    the stored gradients are bf16 numbers; everything stays within the bf16 tolerance of the unrounded step."""
    rng = np.random.default_rng(29)
    n, dims = 60, [8, 10, 4]
    rows, indptr, indices = _small_graph(rng, n, 6)
    Xb = torch.tensor(rng.standard_normal((n, dims[0])), dtype=torch.float32).to(torch.bfloat16)
    bits = Xb.view(torch.int16).numpy().view(np.uint16)
    X64 = Xb.to(torch.float64).numpy()
    y = rng.integers(0, dims[2], size=n).astype(np.int32)
    W = [rng.standard_normal((dims[l], dims[l + 1])) * 0.4 for l in range(2)]
    b = [rng.standard_normal(dims[l + 1]) * 0.1 for l in range(2)]
    seeds = np.array([2, 7, 19, 41, 55, 13], dtype=np.int32)
    ref = orc.gcn_train_step(indptr, indices, bits, y, seeds, [4, 3], W, b, seed=5, step=2, lr=0.1, bf16=True)
    plain = orc.gcn_train_step(indptr, indices, X64.astype(np.float32), y, seeds, [4, 3], W, b, seed=5, step=2, lr=0.1,
                               blocks=ref["blocks"])
    cast = lambda t: t.to(torch.bfloat16).to(torch.float64)
    H = torch.tensor(X64[ref["blocks"][0].src_nodes])
    for l, blk in enumerate(ref["blocks"]):
        s, c, selfw = ref["weights"][l]
        Pm = np.zeros((blk.n_dst, blk.n_src))
        for i in range(blk.n_dst):
            for e in range(blk.indptr[i], blk.indptr[i + 1]):
                Pm[i, blk.cols[e]] += s[i] * c[blk.cols[e]]
            Pm[i, i] += selfw[i]
        A = cast(torch.tensor(Pm) @ H)
        # (the two float64 sums may differ in their last bit, which can move a value across a rounding boundary: then
        # the two results are neighbouring bf16 numbers; that may happen at a few elements, no more)
        off = ref["A"][l] != A.numpy()
        assert off.mean() <= 0.01 and np.all(np.abs(ref["A"][l] - A.numpy())[off] <= 2.0 ** -7 * np.abs(A.numpy())[off])
        Z = torch.tensor(ref["A"][l]) @ cast(torch.tensor(W[l])) + torch.tensor(b[l])
        H = cast(torch.relu(Z)) if l == 0 else Z
        off = ref["H"][l + 1] != H.numpy()
        assert off.mean() <= 0.01 and np.all(np.abs(ref["H"][l + 1] - H.numpy())[off] <= 2.0 ** -7 * np.abs(H.numpy())[off] + 1e-13)
        H = torch.tensor(ref["H"][l + 1])
    def is_bf16(a):
        t = torch.tensor(a)
        return bool(torch.equal(cast(t), t))
    assert is_bf16(ref["A"][0]) and is_bf16(ref["A"][1]) and is_bf16(ref["H"][1]) and is_bf16(ref["dA"][1]) and is_bf16(ref["dH"][1])
    assert not is_bf16(ref["H"][2]) and not is_bf16(ref["dW"][0])          # logits and weight gradients are not rounded
    for k in ("dW", "db", "W_new"):
        for l in range(2):
            assert np.max(np.abs(ref[k][l] - plain[k][l])) <= 2e-2 * np.max(np.abs(plain[k][l])), (k, l)
    assert abs(ref["loss"] - plain["loss"]) <= 2e-2 * abs(plain["loss"])


def test_gat_step_bf16_rounding_points():
    """bf16 storage of the GAT step: the forward equals a float64 computation in which torch's own bf16 cast (an
    independent round-to-nearest-even) is applied to the weights, the projected rows and the hidden activations, with
    the attention written as a dense masked softmax; the stored gradients are bf16 numbers, the logits and the
    parameter gradients are not; everything stays within the bf16 tolerance of the unrounded step."""
    rng = np.random.default_rng(37)
    n, dims = 60, [8, 10, 4]
    rows, indptr, indices = _small_graph(rng, n, 6)
    Xb = torch.tensor(rng.standard_normal((n, dims[0])), dtype=torch.float32).to(torch.bfloat16)
    bits = Xb.view(torch.int16).numpy().view(np.uint16)
    X64 = Xb.to(torch.float64).numpy()
    y = rng.integers(0, dims[2], size=n).astype(np.int32)
    W = [rng.standard_normal((dims[l], dims[l + 1])) * 0.4 for l in range(2)]
    b = [rng.standard_normal(dims[l + 1]) * 0.1 for l in range(2)]
    att = [rng.standard_normal(2 * dims[l + 1]) * 0.5 for l in range(2)]
    seeds = np.array([2, 7, 19, 41, 55, 13], dtype=np.int32)
    ref = orc.gat_train_step(indptr, indices, bits, y, seeds, [4, 3], W, b, att, seed=5, step=2, lr=0.1, bf16=True)
    plain = orc.gat_train_step(indptr, indices, X64.astype(np.float32), y, seeds, [4, 3], W, b, att, seed=5, step=2, lr=0.1,
                               blocks=ref["blocks"])
    cast = lambda t: t.to(torch.bfloat16).to(torch.float64)

    def same_up_to_a_rounding_boundary(mine, other):
        # two float64 sums may differ in their last bit, which can move a value across a rounding boundary: then the
        # results are neighbouring bf16 numbers; that may happen at a few elements, no more
        off = mine != other
        assert off.mean() <= 0.02 and np.all(np.abs(mine - other)[off] <= 2.0 ** -7 * np.abs(other)[off] + 1e-13)

    H = torch.tensor(X64[ref["blocks"][0].src_nodes])
    for l, blk in enumerate(ref["blocks"]):
        F = dims[l + 1]
        z = cast(H @ cast(torch.tensor(W[l])))
        same_up_to_a_rounding_boundary(ref["Z"][l], z.numpy())
        z = torch.tensor(ref["Z"][l])
        # dense attention: logits[i, j] for every source j, minus infinity where there is no edge; duplicates of an
        # edge each count, so the mask holds multiplicities
        mult = np.zeros((blk.n_dst, blk.n_src))
        for i in range(blk.n_dst):
            for e in range(blk.indptr[i], blk.indptr[i + 1]):
                mult[i, blk.cols[e]] += 1
            mult[i, i] += 1
        a_src, a_dst = torch.tensor(att[l][:F]), torch.tensor(att[l][F:])
        score = torch.nn.functional.leaky_relu((z[:blk.n_dst] @ a_dst)[:, None] + (z @ a_src)[None, :], 0.2)
        wgt = torch.tensor(mult) * torch.exp(score - score.max())
        alpha = wgt / wgt.sum(dim=1, keepdim=True)
        pre = alpha @ z + torch.tensor(b[l])
        Hn = cast(torch.relu(pre)) if l == 0 else pre
        if l == 0:
            same_up_to_a_rounding_boundary(ref["H"][l + 1], Hn.numpy())
        else:
            assert np.allclose(ref["H"][l + 1], Hn.numpy(), rtol=1e-11, atol=1e-13)
        H = torch.tensor(ref["H"][l + 1])

    def is_bf16(a):
        t = torch.tensor(a)
        return bool(torch.equal(cast(t), t))
    assert is_bf16(ref["Z"][0]) and is_bf16(ref["Z"][1]) and is_bf16(ref["H"][1])
    assert is_bf16(ref["dz"][0]) and is_bf16(ref["dz"][1]) and is_bf16(ref["dH"][1])
    assert not is_bf16(ref["H"][2]) and not is_bf16(ref["dZ"]) and not is_bf16(ref["dW"][0]) and not is_bf16(ref["datt"][1])
    for k in ("dW", "db", "datt", "W_new", "att_new"):
        for l in range(2):
            assert np.max(np.abs(ref[k][l] - plain[k][l])) <= 3e-2 * np.max(np.abs(plain[k][l])), (k, l)
    assert abs(ref["loss"] - plain["loss"]) <= 2e-2 * abs(plain["loss"])


# ----------------------------------------------------------------- Adam
def test_adam_matches_library_optimiser():
    rng = np.random.default_rng(31)
    w0 = rng.standard_normal((7, 5))
    grads = [rng.standard_normal((7, 5)) * s for s in (1.0, 0.1, 3.0, 1e-4)]
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.Adam([p], lr=0.02, betas=(0.8, 0.95), eps=1e-7)
    w, m, v = w0, np.zeros_like(w0), np.zeros_like(w0)
    for t, g in enumerate(grads, start=1):
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, m, v = orc.adam(w, g, m, v, t, 0.02, 0.8, 0.95, 1e-7)
        assert np.allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-14)
    # first update from zero moments: a step of lr * sign(g) (up to eps)
    w1, _, _ = orc.adam(np.zeros(4), np.array([2.0, -3.0, 0.5, -1e-3]), np.zeros(4), np.zeros(4), 1, 0.1)
    assert np.allclose(w1, [-0.1, 0.1, -0.1, 0.1], rtol=1e-4)


# ----------------------------------------------------------------- GAT attention aggregation
def test_gat_aggregate_matches_autograd_and_closed_forms():
    rng = np.random.default_rng(41)
    n, F = 60, 6
    rows, indptr, indices = _small_graph(rng, n, 7)
    dst = rng.choice(n, size=15, replace=False).astype(np.int32)
    blk = orc.sample_block(indptr, indices, dst, 4, 2, 0, 1)
    z = rng.standard_normal((blk.n_src, F))
    a_src, a_dst = rng.standard_normal(F), rng.standard_normal(F)
    g = rng.standard_normal((blk.n_dst, F))
    out, alpha, alpha_self = orc.gat_aggregate_fwd(blk.indptr, blk.cols, z, a_src, a_dst)
    # every row's attention (edges + self edge) sums to one
    for i in range(blk.n_dst):
        assert abs(alpha[blk.indptr[i]:blk.indptr[i + 1]].sum() + alpha_self[i] - 1.0) < 1e-14
    # zero attention vectors: uniform attention = plain mean over the neighbours and the node itself
    out0, _, _ = orc.gat_aggregate_fwd(blk.indptr, blk.cols, z, 0 * a_src, 0 * a_dst)
    for i in range(blk.n_dst):
        c = list(blk.cols[blk.indptr[i]:blk.indptr[i + 1]]) + [i]
        assert np.allclose(out0[i], z[c].mean(axis=0))
    # independent formulation in torch (float64) with autograd
    zt = torch.tensor(z, requires_grad=True)
    at, bt = torch.tensor(a_src, requires_grad=True), torch.tensor(a_dst, requires_grad=True)
    outs = []
    for i in range(blk.n_dst):
        c = torch.tensor(list(blk.cols[blk.indptr[i]:blk.indptr[i + 1]]) + [i], dtype=torch.long)
        s = torch.nn.functional.leaky_relu(zt[i] @ bt + zt[c] @ at, 0.2)
        outs.append(torch.softmax(s, 0) @ zt[c])
    ot = torch.stack(outs)
    assert np.allclose(out, ot.detach().numpy(), rtol=1e-12, atol=1e-13)
    (ot * torch.tensor(g)).sum().backward()
    dz, da_src, da_dst = orc.gat_aggregate_bwd(blk.indptr, blk.cols, z, a_src, a_dst, g)
    assert np.allclose(dz, zt.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(da_src, at.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(da_dst, bt.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_gat_step_gradients_match_autograd_and_central_differences():
    rng = np.random.default_rng(43)
    n, dims = 40, [5, 6, 3]
    rows, indptr, indices = _small_graph(rng, n, 5)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    y = rng.integers(0, dims[2], size=n).astype(np.int32)
    W = [rng.standard_normal((dims[l], dims[l + 1])) * 0.5 for l in range(2)]
    b = [rng.standard_normal(dims[l + 1]) * 0.2 for l in range(2)]
    att = [rng.standard_normal(2 * dims[l + 1]) * 0.6 for l in range(2)]
    seeds = np.array([2, 7, 19, 31, 11, 0], dtype=np.int32)
    ref = orc.gat_train_step(indptr, indices, X, y, seeds, [3, 2], W, b, att, seed=4, step=2, lr=0.05)
    blocks = ref["blocks"]

    def model(Wt, bt, at):   # the same model row by row in torch (float64)
        H = torch.tensor(X[blocks[0].src_nodes].astype(np.float64))
        for l, blk in enumerate(blocks):
            F = dims[l + 1]
            z = H @ Wt[l]
            outs = []
            for i in range(blk.n_dst):
                c = torch.tensor(list(blk.cols[blk.indptr[i]:blk.indptr[i + 1]]) + [i], dtype=torch.long)
                s = torch.nn.functional.leaky_relu(z[i] @ at[l][F:] + z[c] @ at[l][:F], 0.2)
                outs.append(torch.softmax(s, 0) @ z[c])
            pre = torch.stack(outs) + bt[l]
            H = torch.relu(pre) if l == 0 else pre
        return torch.nn.functional.cross_entropy(H, torch.tensor(y[seeds].astype(np.int64)))

    Wt = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in W]
    bt = [torch.tensor(v, dtype=torch.float64, requires_grad=True) for v in b]
    at = [torch.tensor(v, dtype=torch.float64, requires_grad=True) for v in att]
    loss = model(Wt, bt, at)
    loss.backward()
    assert abs(loss.item() - ref["loss"]) < 1e-12
    for l in range(2):
        assert np.allclose(ref["dW"][l], Wt[l].grad.numpy(), rtol=1e-10, atol=1e-12)
        assert np.allclose(ref["db"][l], bt[l].grad.numpy(), rtol=1e-10, atol=1e-12)
        assert np.allclose(ref["datt"][l], at[l].grad.numpy(), rtol=1e-10, atol=1e-12)
        assert np.allclose(ref["att_new"][l], att[l] - 0.05 * at[l].grad.numpy(), rtol=1e-12, atol=1e-13)
        assert np.allclose(ref["W_new"][l], W[l] - 0.05 * Wt[l].grad.numpy(), rtol=1e-12, atol=1e-13)
    # central differences of the oracle's own loss on a few coordinates of every parameter
    h = 1e-6
    for l in range(2):
        for P, G in ((W, ref["dW"]), (b, ref["db"]), (att, ref["datt"])):
            flat, g = P[l].reshape(-1), G[l].reshape(-1)
            for idx in range(0, flat.size, max(1, flat.size // 5)):
                keep = flat[idx]
                flat[idx] = keep + h
                lp = orc.gat_train_step(indptr, indices, X, y, seeds, [3, 2], W, b, att, 4, 2, 0.0, blocks=blocks)["loss"]
                flat[idx] = keep - h
                lm = orc.gat_train_step(indptr, indices, X, y, seeds, [3, 2], W, b, att, 4, 2, 0.0, blocks=blocks)["loss"]
                flat[idx] = keep
                assert abs((lp - lm) / (2 * h) - g[idx]) <= 1e-6 * max(1.0, abs(g[idx])) + 1e-8, (l, idx)
