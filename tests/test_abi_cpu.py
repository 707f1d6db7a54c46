"""CPU-only checks of the boundary: the library loads, exports every symbol the
header declares, and its argument validation (forced from the host through a
GPU-less context) returns the documented codes."""
import os
import re

import pytest

from paper_2305_02522_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "bitgnn.h")).read()
    declared = set(re.findall(r"\b(bitgnn_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 31
    assert declared == set(B.EXPORTS)
    import ctypes
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert getattr(lib, name) is not None


@pytest.fixture()
def vctx():
    ctx = B.Context(-1)
    yield ctx
    ctx.close()


def _code(fn, *a):
    with pytest.raises(B.BitgnnError) as e:
        fn(*a)
    return e.value.code


P8 = 0x1000       # fake, aligned, never dereferenced: validation contexts do not launch


def test_pack_validation(vctx):
    assert _code(B.pack_f32, vctx, P8, 4, 100, 100, None, P8, 2) == B.ERR_NO_DEVICE
    assert "no GPU" in vctx.last_error()
    assert _code(B.pack_f32, vctx, P8, 4, 100, 99, None, P8, 2) == B.ERR_INVALID_ARG   # ldx < K
    assert _code(B.pack_f32, vctx, P8, 4, 100, 100, None, P8, 1) == B.ERR_INVALID_ARG  # stride
    assert _code(B.pack_f32, vctx, None, 4, 100, 100, None, P8, 2) == B.ERR_INVALID_ARG
    assert _code(B.pack_f32, vctx, P8, 4, 0, 100, None, P8, 2) == B.ERR_INVALID_ARG
    assert _code(B.pack_f32, vctx, P8 + 2, 4, 100, 100, None, P8, 2) == B.ERR_ALIGNMENT
    assert _code(B.pack_f32, vctx, P8, 4, 100, 100, None, P8 + 4, 2) == B.ERR_ALIGNMENT
    assert _code(B.pack_i8, vctx, P8 + 1, 4, 100, 100, P8, 2) == B.ERR_NO_DEVICE      # bytes: any
    B.pack_f32(vctx, None, 0, 100, 100, None, None, 2)                                 # n = 0: no-op
    assert _code(B.pack_weights_i8, vctx, P8, 10, 4, 3, P8, 1) == B.ERR_INVALID_ARG    # ldw < M


def test_adj_build_validation(vctx):
    assert _code(B.adj_build, vctx, P8, P8, 10, 5, 3) == B.ERR_NO_DEVICE
    assert _code(B.adj_build, vctx, P8, P8, 10, 0, 0) == B.ERR_INVALID_ARG
    assert _code(B.adj_build, vctx, P8, P8, -1, 5, 0) == B.ERR_INVALID_ARG
    assert _code(B.adj_build, vctx, P8, P8, 10, 5, 4) == B.ERR_INVALID_ARG             # flags
    assert _code(B.adj_build, vctx, None, P8, 10, 5, 0) == B.ERR_INVALID_ARG
    assert _code(B.adj_build, vctx, P8 + 2, P8, 10, 5, 0) == B.ERR_ALIGNMENT
    assert _code(B.adj_build, vctx, P8, P8, 1 << 30, 5, 1) == B.ERR_RANGE              # 2E+N >= 2^31


def test_bgemm_validation(vctx):
    ok = (P8, 10, 2, 100, 2, P8, 7, 2)
    assert _code(B.bgemm, vctx, *ok, B.EPI_THRESH_BITS, P8, None, P8, 1) == B.ERR_NO_DEVICE
    assert _code(B.bgemm, vctx, *ok, B.EPI_THRESH_BITS, None, None, P8, 1) == B.ERR_INVALID_ARG
    assert _code(B.bgemm, vctx, *ok, B.EPI_SCALE_F32, None, None, P8, 7) == B.ERR_INVALID_ARG
    assert _code(B.bgemm, vctx, *ok, B.EPI_RAW_I32, None, None, P8, 6) == B.ERR_INVALID_ARG
    assert _code(B.bgemm, vctx, *ok, 3, None, None, P8, 7) == B.ERR_INVALID_ARG
    assert _code(B.bgemm, vctx, P8, 10, 1, 100, 2, P8, 7, 2, 0, None, None, P8, 7) == \
        B.ERR_INVALID_ARG                                                              # x_stride
    assert _code(B.bgemm, vctx, P8, 10, 2, 129, 2, P8, 7, 2, 0, None, None, P8, 7) == \
        B.ERR_INVALID_ARG                                                              # K > bits
    assert _code(B.bgemm, vctx, P8 + 4, 10, 2, 100, 2, P8, 7, 2, 0, None, None, P8, 7) == \
        B.ERR_ALIGNMENT
    assert _code(B.bgemm, vctx, *ok, B.EPI_THRESH_BITS, P8, None, P8 + 4, 1) == B.ERR_ALIGNMENT
    assert _code(B.bgemm, vctx, *ok, B.EPI_RAW_I32, None, None, P8 + 4, 7) == B.ERR_NO_DEVICE


def test_aggregation_and_layer_validation(vctx):
    assert _code(B.bspmm, vctx, None, P8, 64, 1, B.EPI_THRESH_BITS, P8, P8, 1) == B.ERR_INVALID_ARG
    assert _code(B.spmm_i32, vctx, None, P8, 7, 7, 64, None, P8, 7) == B.ERR_INVALID_ARG
    assert _code(B.adj_tune, vctx, None, 128, 3) == B.ERR_INVALID_ARG
    assert _code(B.spmm_f32, vctx, None, P8, 0, 7, 7, None, None, B.EPI_SCALE_F32, None, P8,
                 7) == B.ERR_INVALID_ARG
    assert _code(B.gcn_layer, vctx, None, P8, 2, 100, 2, P8, 64, 2, P8, P8, P8, P8, 1) == \
        B.ERR_INVALID_ARG
    assert _code(B.gcn_out_layer, vctx, None, P8, 2, 100, 2, P8, 7, 2, P8, P8, P8, 7) == \
        B.ERR_INVALID_ARG
    assert _code(B.sage_layer, vctx, None, P8, 100, P8, 64, 4, P8, P8, P8, 2) == B.ERR_INVALID_ARG
    assert _code(B.sage_layer_weighted, vctx, None, P8, 100, P8, 64, 4, P8, None, P8, P8, P8,
                 2) == B.ERR_INVALID_ARG
    assert _code(B.gcn_out_layer_weighted, vctx, None, P8, 2, 100, 2, P8, 7, 2, P8, P8, P8, P8,
                 P8, 7) == B.ERR_INVALID_ARG
    assert _code(B.gcn_layer_weighted, vctx, None, P8, 2, 100, 2, P8, 64, 2, P8, P8, P8, P8, P8,
                 P8, 1) == B.ERR_INVALID_ARG
    assert _code(B.sage_out_layer, vctx, None, P8, 100, P8, 7, 4, P8, P8, P8, 7) == \
        B.ERR_INVALID_ARG
    assert _code(B.spmm_i16, vctx, None, P8, 7, 8, P8, None, None, B.EPI_SCALE_F32, None, P8,
                 7) == B.ERR_INVALID_ARG
    assert _code(B.gcn_layer_full, vctx, None, P8, 2, 100, 2, P8, 64, 2, P8, P8, P8, P8, P8, P8,
                 1) == B.ERR_INVALID_ARG
    assert _code(B.gcn_layer_full_f32, vctx, None, P8, 100, 100, None, P8, 64, 2, P8, P8, P8, P8,
                 P8, P8, 1) == B.ERR_INVALID_ARG
    assert _code(B.add, vctx, P8, False, 70, P8, True, 2, 4, 70, B.EPI_SCALE_F32, None, P8,
                 70) == B.ERR_NO_DEVICE
    assert _code(B.add, vctx, P8, False, 70, P8, True, 1, 4, 70, B.EPI_SCALE_F32, None, P8,
                 70) == B.ERR_INVALID_ARG
    assert _code(B.gcn2_fused, vctx, None, P8, 100, 100, P8, 64, 2, P8, P8, P8, 7, 1, P8, P8, P8,
                 1, P8, 7) == B.ERR_INVALID_ARG


def test_fused_spin_limit_validation(vctx):
    B.ctx_set_fused_spin_limit(vctx, 1)
    B.ctx_set_fused_spin_limit(vctx, 1 << 22)
    assert _code(B.ctx_set_fused_spin_limit, vctx, 0) == B.ERR_INVALID_ARG


def test_chain_check_types_the_papers_recipes(vctx):
    """The two recipes of Table 3's caption and the GCN pairs of Section 3.1.2 are well
    typed; a precision mismatch, a full-precision weight operand and malformed names are
    reported at their position."""
    ok = ["MM.FBB + BSpMM.BBB + MM.BBF + BSpMM.FBF",          # binary aggregation
          "BMM.FBF BSpMM.FBB BMM.BBF BSpMM.FBF",              # full-precision aggregation
          "BMM.BBB,BSpMM.BBF", "BSpMM.BBB > ADD.BBF > BMM.FBB", "ADD.FFF"]
    for chain in ok:
        assert B.chain_check(vctx, chain) == -1, chain
    assert B.chain_check(vctx, "MM.FBB BSpMM.FBB") == 1
    assert "takes F but its predecessor produces B" in vctx.last_error()
    assert B.chain_check(vctx, "BMM.FBB BSpMM.BBB BMM.FBF") == 2
    assert B.chain_check(vctx, "BMM.FFB") == 0 and "weight" in vctx.last_error()
    assert B.chain_check(vctx, "BMM.FBB BSpMM.BFB") == 1 and "adjacency" in vctx.last_error()
    assert B.chain_check(vctx, "BMM.FBB CONV.BBB") == 1
    assert B.chain_check(vctx, "BMM.FB") == 0
    assert B.chain_check(vctx, "BMM.FBBB") == 0
    assert B.chain_check(vctx, "BMM.FXB") == 0
    with pytest.raises(B.BitgnnError):
        B.chain_check(vctx, "  ")
    assert _code(B.gcn_layer_tune, vctx, None, 64, 64, 3) == B.ERR_INVALID_ARG


def test_workspace_and_bgemm_path_calls(vctx):
    """The set-up calls of the workspace contract and the BMM kernel choice validate on the
    host: no compute call allocates, so a caller sizes and reserves the workspace first."""
    assert _code(B.adj_workspace_bytes, vctx, None, 128, 41) == B.ERR_INVALID_ARG   # no handle
    assert _code(B.ctx_reserve, vctx, 1 << 20) == B.ERR_NO_DEVICE
    assert B.ctx_workspace(vctx) == 0
    assert _code(B.ctx_set_bgemm_path, vctx, 3) == B.ERR_INVALID_ARG
    assert _code(B.ctx_set_bgemm_path, vctx, -1) == B.ERR_INVALID_ARG
    # the choice is a host-side rule: matrix cores from 65,536 rows on when the weights fit
    assert B.ctx_bgemm_kernel(vctx, 1000, 2, 128) == B.BGEMM_VALU
    assert B.ctx_bgemm_kernel(vctx, 232965, 2, 128) == B.BGEMM_MFMA
    assert B.ctx_bgemm_kernel(vctx, 232965, 32, 128) == B.BGEMM_VALU     # K = 2048: not in LDS
    assert B.ctx_bgemm_kernel(vctx, 232965, 16, 256) == B.BGEMM_MFMA     # K = 1024: column chunks,
    assert B.ctx_bgemm_kernel(vctx, 89250, 16, 256) == B.BGEMM_VALU      # from 131,072 rows on
    assert B.ctx_bgemm_kernel(vctx, 89250, 8, 7) == B.BGEMM_MFMA         # 16 padded columns fit
    B.ctx_set_bgemm_path(vctx, B.BGEMM_VALU)
    assert B.ctx_bgemm_kernel(vctx, 232965, 2, 128) == B.BGEMM_VALU
    B.ctx_set_bgemm_path(vctx, B.BGEMM_MFMA)
    assert B.ctx_bgemm_kernel(vctx, 1000, 2, 128) == B.BGEMM_MFMA
    B.ctx_set_bgemm_path(vctx, B.BGEMM_AUTO)
    assert _code(B.ctx_bgemm_kernel, vctx, 10, 0, 5) == B.ERR_INVALID_ARG
    assert B.ERR_WORKSPACE == -8


def test_ctx_create_rejects_bad_device():
    with pytest.raises(B.BitgnnError):
        B.Context(-2)


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU only and says so before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr
