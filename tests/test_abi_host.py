"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, and its pure-host queries and argument
validation behave."""
import ctypes
import os
import re

import pytest

from paper_2404_02300_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    hdr = open(os.path.join(ROOT, "include", "sdt.h")).read()
    return sorted(set(re.findall(r"\b(sdt_[a-z_0-9]+)\s*\(", hdr)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = _declared()
    assert len(names) >= 13
    for n in names:
        assert hasattr(L, n), n
        assert n in B.EXPORTS, f"binding lacks {n}"
    assert re.fullmatch(r"\d+\.\d+\.\d+", B.sdt_version())


def test_binding_mirrors_header_names():
    for n in _declared():
        assert hasattr(B, n), n


def test_struct_mirrors_have_the_library_sizes():
    for which, cls in enumerate([B.sdt_csr, B.sdt_block, B.sdt_model, B.sdt_step_layout, B.sdt_partition]):
        assert B.sdt_struct_bytes(which) == ctypes.sizeof(cls), cls.__name__
    assert B.sdt_struct_bytes(99) == 0


def test_model_kinds_layouts_and_their_argument_checks():
    f = [10, 5]
    sage = B.sdt_train_step_layout(1 << 14, 256, f, _model([602, 64, 8]), B.SDT_F32)
    assert sage.ld_in == 608 and sage.t_indptr[0] == 0 and sage.t_indptr[1] != 0    # input rows on whole 128-byte lines
    assert B.sdt_train_step_layout(1 << 14, 256, f, _model([64, 64, 8]), B.SDT_F32).ld_in == 64
    assert B.sdt_train_step_layout(1 << 14, 256, f, _model([100, 64, 8]), B.SDT_BF16).ld_in == 128
    gat = _model([64, 64, 8])
    gat.kind, gat.gat_slope = B.SDT_MODEL_GAT, 0.2
    lay = B.sdt_train_step_layout(1 << 14, 256, f, gat, B.SDT_F32)
    assert lay.ld_in == 64 and lay.t_indptr[0] != 0 and lay.z[0] != 0 and lay.dz[1] != 0 and lay.gatws[0] != 0
    assert lay.A[0] == 0 and lay.dH[0] == 0 and lay.dH[1] != 0
    gcn = _model([64, 64, 8])
    gcn.kind = B.SDT_MODEL_GCN
    assert B.sdt_train_step_layout(1 << 14, 256, f, gcn, B.SDT_F32).norm[1] != 0
    for bad_kind in (B.SDT_MODEL_GCN, B.SDT_MODEL_GAT):
        m = _model([63, 64, 8])      # odd input width: the single-matrix kinds split a row into two halves
        m.kind, m.gat_slope = bad_kind, 0.2
        with pytest.raises(B.SdtError):
            B.sdt_train_step_layout(1 << 14, 256, f, m, B.SDT_F32)
    gcn16 = B.sdt_train_step_layout(1 << 14, 256, f, gcn, B.SDT_BF16)     # GCN: fp32 or bf16 storage
    assert gcn16.norm[1] != 0 and gcn16.total_bytes < B.sdt_train_step_layout(1 << 14, 256, f, gcn, B.SDT_F32).total_bytes
    gat16 = B.sdt_train_step_layout(1 << 14, 256, f, gat, B.SDT_BF16)     # GAT likewise
    assert gat16.z[0] != 0 and gat16.total_bytes < lay.total_bytes
    gat.gat_slope = 1.5
    with pytest.raises(B.SdtError):
        B.sdt_train_step_layout(1 << 14, 256, f, gat, B.SDT_F32)
    unknown = _model([64, 64, 8])
    unknown.kind = 7
    with pytest.raises(B.SdtError):
        B.sdt_train_step_layout(1 << 14, 256, f, unknown, B.SDT_F32)


def test_workspace_queries_are_host_arithmetic():
    a = B.sdt_sample_workspace_bytes(1 << 21, 1024, 10)
    b = B.sdt_sample_workspace_bytes(1 << 21, 11264, 15)
    assert 0 < a < b
    assert a >= (1 << 21) * 4 + (1 << 21) // 2            # id map + two state bits and a rank word per 16 nodes
    assert B.sdt_sample_workspace_bytes(-1, 4, 4) == 0
    assert B.sdt_linear_bwd_workspace_bytes(11264, 100, 256) >= 2 * 100 * 256 * 4


def _model(dims):
    m = B.sdt_model()
    m.n_layers = len(dims) - 1
    for i, d in enumerate(dims):
        m.dims[i] = d
    return m


def test_step_layout_bounds_match_the_frontier_recurrence():
    lay = B.sdt_train_step_layout(1 << 21, 1024, [15, 10], _model([100, 256, 47]), B.SDT_F32)
    assert list(lay.cap_dst[:2]) == [11264, 1024]
    assert list(lay.cap_nnz[:2]) == [168960, 10240]
    assert list(lay.cap_src[:2]) == [180224, 11264]
    lay4 = B.sdt_train_step_layout(1 << 24, 1024, [15, 10, 5], _model([128, 256, 256, 172]), B.SDT_BF16)
    assert list(lay4.cap_dst[:3]) == [67584, 6144, 1024] and lay4.cap_src[0] == 1081344
    # the frontier can never exceed the partition
    small = B.sdt_train_step_layout(1 << 14, 256, [10, 5], _model([64, 64, 8]), B.SDT_F32)
    assert small.cap_src[0] == 1 << 14 and small.cap_dst[0] == 1536
    offs = [small.counts[0], small.indptr[0], small.cols[0], small.src_nodes[0], small.H[0], small.H[1], small.H[2],
            small.A[0], small.A[1], small.dZ, small.scratch]
    assert len(set(offs)) == len(offs) and max(offs) < small.total_bytes
    assert all(o % 256 == 0 for o in offs)


def test_invalid_arguments_are_reported_not_crashed():
    f = (ctypes.c_int32 * 2)(10, 5)
    lay = B.sdt_step_layout()
    L = B.lib()
    m = _model([64, 64, 8])
    assert L.sdt_train_step_layout(1 << 14, 256, f, ctypes.byref(m), 7, ctypes.byref(lay)) == B.SDT_ERR_INVALID_ARG
    assert "dtype" in B.sdt_last_error()
    bad = (ctypes.c_int32 * 2)(10, 65)
    assert L.sdt_train_step_layout(1 << 14, 256, bad, ctypes.byref(m), 0, ctypes.byref(lay)) == B.SDT_ERR_INVALID_ARG
    assert L.sdt_train_step_layout(100, 256, f, ctypes.byref(m), 0, ctypes.byref(lay)) == B.SDT_ERR_INVALID_ARG
    m.n_layers = 9
    assert L.sdt_train_step_layout(1 << 14, 256, f, ctypes.byref(m), 0, ctypes.byref(lay)) == B.SDT_ERR_INVALID_ARG
    with pytest.raises(B.SdtError):
        B.sdt_train_step_layout(1 << 14, 256, [10, 5], m, 0)
    # null graph / null block are rejected before any launch
    assert L.sdt_sample_csr(None, None, 0, None, 4, 0, 0, 0, None, None, 0, None) == B.SDT_ERR_INVALID_ARG
    assert L.sdt_sage_aggregate_fwd(None, None, 0, 4, 0, None, 0, None) == B.SDT_ERR_INVALID_ARG
    assert L.sdt_gather_features(None, 4, 8, 0, None, 3, None, None, 8, None) == B.SDT_ERR_INVALID_ARG
    assert L.sdt_sage_linear_fwd(None, 4, None, 4, 3, None, 4, 4, None, None, 0, 0, None, 4, 0, None) == B.SDT_ERR_INVALID_ARG


def test_noalloc_entry_point_rejects_oversized_shapes_on_the_host():
    """The size check of the entry point with built-in scratch is host arithmetic and comes before any GPU call."""
    L = B.lib()
    n, fin, fout = 67584, 128, 256
    assert B.sdt_linear_bwd_workspace_bytes(n, fin, fout) > B.SDT_NOALLOC_SCRATCH_BYTES
    rc = L.sdt_sage_linear_bwd_noalloc(None, fout, 0, None, 0, 0, None, fin, None, fin, n, None, fin, fout, None, 0, None, None,
                                       None, None, 0, None)
    assert rc == B.SDT_ERR_WORKSPACE and "built-in" in B.sdt_last_error()
    assert L.sdt_sage_linear_bwd_noalloc(None, 4, 0, None, 0, 0, None, 4, None, 4, -1, None, 4, 4, None, 0, None, None,
                                         None, None, 0, None) == B.SDT_ERR_INVALID_ARG


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU's throughput; asking for more exits with a message before anything is loaded."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
