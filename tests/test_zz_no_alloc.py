"""The entry point that allocates nothing (sdt_sage_linear_bwd_noalloc: scratch in a device array
built into the library) against the entry point it is a variant of (sdt_sage_linear_bwd with a
caller's workspace), through the C ABI: two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_2404_02300_amd import binding as B

pytestmark = pytest.mark.gpu


def _case(rng, n, fin, fout, bf16, relu):
    dt = torch.bfloat16 if bf16 else torch.float32
    t = lambda *shape: torch.from_numpy(rng.standard_normal(shape).astype(np.float32))
    Hs, A = t(n + 3, fin).to(dt).cuda(), t(n, fin).to(dt).cuda()
    W = (t(2 * fin, fout) / np.sqrt(2 * fin)).cuda()
    Y = t(n, fout).to(dt).cuda() if relu else None
    dY = t(n, fout).to(dt if relu else torch.float32).cuda()
    return dt, Hs, A, W, Y, dY


def _both(rng, n, fin, fout, bf16, relu, with_inputs=True, n_d=None):
    dt, Hs, A, W, Y, dY = _case(rng, n, fin, fout, bf16, relu)
    outs = []
    for noalloc in (False, True):
        dW = torch.full((2 * fin, fout), float("nan"), dtype=torch.float32, device="cuda")
        db = torch.full((fout,), float("nan"), dtype=torch.float32, device="cuda")
        dS = torch.zeros(n, fin, dtype=dt, device="cuda") if with_inputs else None
        dA = torch.zeros(n, fin, dtype=dt, device="cuda") if with_inputs else None
        if noalloc:
            B.sdt_sage_linear_bwd_noalloc(dY, Y, relu, Hs, A, W, dW, db, dS, dA, n_d=n_d)
        else:
            ws = torch.empty(B.sdt_linear_bwd_workspace_bytes(n, fin, fout), dtype=torch.uint8, device="cuda")
            B.sdt_sage_linear_bwd(dY, Y, relu, Hs, A, W, dW, db, dS, dA, ws, n_d=n_d)
        torch.cuda.synchronize()
        outs.append((dW, db, dS, dA))
    for got, want, name in zip(outs[1], outs[0], ("dW", "db", "dSelf", "dAgg")):
        if want is None:
            continue
        assert torch.isfinite(want.float()).all(), name
        assert torch.equal(got, want), f"{name}: n={n} in={fin} out={fout} bf16={bf16} relu={relu}"


def test_noalloc_matches_workspace_entry_point_two_calls_second_smaller():
    print("no-alloc projection backward: large call, then a smaller one", flush=True)
    rng = np.random.default_rng(5)
    # large first (several row splits, masked copy in use), then smaller inputs that reuse the same scratch
    _both(rng, 11264, 100, 256, False, True)
    _both(rng, 1000, 64, 41, False, True)
    _both(rng, 333, 70, 41, False, False, with_inputs=False)
    _both(rng, 700, 128, 256, True, True)
    _both(rng, 129, 256, 172, True, False)
    # device-side row count below the bound, after a call that used more rows
    n_d = torch.tensor([77], dtype=torch.int32, device="cuda")
    _both(rng, 500, 32, 48, False, True, n_d=n_d)


def test_noalloc_rejects_shapes_beyond_the_built_in_scratch():
    n, fin, fout = 67584, 128, 256
    assert B.sdt_linear_bwd_workspace_bytes(n, fin, fout) > B.SDT_NOALLOC_SCRATCH_BYTES
    z = torch.zeros(1, dtype=torch.float32, device="cuda")
    A = torch.zeros(n, fin, dtype=torch.float32, device="cuda")
    dY = torch.zeros(n, fout, dtype=torch.float32, device="cuda")
    W = torch.zeros(2 * fin, fout, dtype=torch.float32, device="cuda")
    dW, db = torch.zeros_like(W), torch.zeros(fout, dtype=torch.float32, device="cuda")
    with pytest.raises(B.SdtError) as e:
        B.sdt_sage_linear_bwd_noalloc(dY, None, False, A, A, W, dW, db, None, None)
    assert e.value.code == B.SDT_ERR_WORKSPACE and "built-in" in str(e.value)
    del z
