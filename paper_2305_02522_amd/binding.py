"""ctypes binding of libbitgnn.so: same entry points as include/bitgnn.h, argument
marshalling only.  torch tensors provide device memory and the stream; every
step of the computation runs in the library's HIP kernels.  There is no CPU
path: if the library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbitgnn.so")

OK = 0
ERR_INVALID_ARG = -1
ERR_ALIGNMENT = -2
ERR_INDEX_RANGE = -3
ERR_RANGE = -4
ERR_HIP = -5
ERR_UNSUPPORTED = -6
ERR_NO_DEVICE = -7
ERR_WORKSPACE = -8

BGEMM_AUTO, BGEMM_VALU, BGEMM_MFMA = 0, 1, 2

ADJ_SYMMETRIZE = 1
ADJ_ADD_SELF_LOOPS = 2

EPI_RAW_I32 = 0
EPI_THRESH_BITS = 1
EPI_SCALE_F32 = 2

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} not found: build it with `python -m paper_2305_02522_amd.build` "
        "(there is no fallback implementation)")

_lib = ctypes.CDLL(LIB_PATH)

_vp, _i64, _i32, _u32, _int = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32,
                               ctypes.c_int)

_SIGNATURES = {
    "bitgnn_ctx_create": (_int, [ctypes.POINTER(_vp), _int]),
    "bitgnn_ctx_destroy": (None, [_vp]),
    "bitgnn_last_error": (ctypes.c_char_p, [_vp]),
    "bitgnn_ctx_set_tuning": (_int, [_vp, _i32, _i32, _i32]),
    "bitgnn_ctx_set_bgemm_path": (_int, [_vp, _int]),
    "bitgnn_ctx_bgemm_kernel": (_int, [_vp, _i64, _i32, _i32, ctypes.POINTER(_int)]),
    "bitgnn_ctx_reserve": (_int, [_vp, ctypes.c_size_t]),
    "bitgnn_ctx_workspace": (_int, [_vp, ctypes.POINTER(ctypes.c_size_t)]),
    "bitgnn_adj_workspace_bytes": (_int, [_vp, _i32, _i32, ctypes.POINTER(ctypes.c_size_t)]),
    "bitgnn_ctx_kernel_timing": (_int, [_vp, _int]),
    "bitgnn_ctx_kernel_times": (_int, [_vp, ctypes.POINTER(ctypes.c_float), _i32,
                                       ctypes.POINTER(_i32)]),
    "bitgnn_pack_f32": (_int, [_vp, _vp, _vp, _i64, _i32, _i64, _vp, _vp, _i64]),
    "bitgnn_pack_i8": (_int, [_vp, _vp, _vp, _i64, _i32, _i64, _vp, _i64]),
    "bitgnn_pack_weights_i8": (_int, [_vp, _vp, _vp, _i32, _i32, _i64, _vp, _i64]),
    "bitgnn_adj_build": (_int, [_vp, _vp, _vp, _vp, _i64, _i64, _u32, ctypes.POINTER(_vp)]),
    "bitgnn_adj_info": (_int, [_vp, ctypes.POINTER(_i64), ctypes.POINTER(_i64),
                               ctypes.POINTER(_i64), ctypes.POINTER(ctypes.c_size_t)]),
    "bitgnn_adj_csr": (_int, [_vp, ctypes.POINTER(_vp), ctypes.POINTER(_vp), ctypes.POINTER(_vp)]),
    "bitgnn_adj_blocked_info": (_int, [_vp] + [ctypes.POINTER(_i64)] * 6),
    "bitgnn_adj_destroy": (None, [_vp]),
    "bitgnn_bgemm": (_int, [_vp, _vp, _vp, _i64, _i64, _i32, _i32, _vp, _i32, _i64, _int, _vp,
                            _vp, _vp, _i64]),
    "bitgnn_bgemm_f32": (_int, [_vp, _vp, _vp, _i64, _i32, _i64, _vp, _vp, _i32, _i64, _int, _vp,
                                _vp, _vp, _i64]),
    "bitgnn_gcn_layer_f32": (_int, [_vp, _vp, _vp, _vp, _i32, _i64, _vp, _vp, _i32, _i64, _vp, _vp,
                                    _vp, _vp, _i64]),
    "bitgnn_adj_tune": (_int, [_vp, _vp, _vp, _i32, _i32, _vp, _vp]),
    "bitgnn_bspmm": (_int, [_vp, _vp, _vp, _vp, _i32, _i64, _int, _vp, _vp, _i64]),
    "bitgnn_bspmm_static": (_int, [_vp, _vp, _vp, _vp, _i32, _i64, _int, _vp, _vp, _i64]),
    "bitgnn_spmm_i32": (_int, [_vp, _vp, _vp, _vp, _i32, _i64, _i64, _vp, _vp, _i64]),
    "bitgnn_spmm_f32": (_int, [_vp, _vp, _vp, _vp, _int, _i32, _i64, _vp, _vp, _int, _vp, _vp,
                               _i64]),
    "bitgnn_spmm_i16": (_int, [_vp, _vp, _vp, _vp, _i32, _i64, _vp, _vp, _vp, _int, _vp, _vp, _i64]),
    "bitgnn_add": (_int, [_vp, _vp, _vp, _int, _i64, _vp, _int, _i64, _i64, _i32, _int, _vp, _vp,
                          _i64]),
    "bitgnn_gcn_layer": (_int, [_vp, _vp, _vp, _vp, _i64, _i32, _i32, _vp, _i32, _i64, _vp, _vp,
                                _vp, _vp, _i64]),
    "bitgnn_gcn_out_layer": (_int, [_vp, _vp, _vp, _vp, _i64, _i32, _i32, _vp, _i32, _i64, _vp,
                                    _vp, _vp, _i64]),
    "bitgnn_sage_layer": (_int, [_vp, _vp, _vp, _vp, _i32, _vp, _i32, _i64, _vp, _vp, _vp, _i64]),
    "bitgnn_sage_out_layer": (_int, [_vp, _vp, _vp, _vp, _i32, _vp, _i32, _i64, _vp, _vp, _vp,
                                     _i64]),
    "bitgnn_gcn_layer_weighted": (_int, [_vp, _vp, _vp, _vp, _i64, _i32, _i32, _vp, _i32, _i64,
                                         _vp, _vp, _vp, _vp, _vp, _vp, _i64]),
    "bitgnn_gcn_out_layer_weighted": (_int, [_vp, _vp, _vp, _vp, _i64, _i32, _i32, _vp, _i32, _i64,
                                             _vp, _vp, _vp, _vp, _vp, _i64]),
    "bitgnn_sage_layer_weighted": (_int, [_vp, _vp, _vp, _vp, _i32, _vp, _i32, _i64, _vp, _vp,
                                          _vp, _vp, _vp, _i64]),
    "bitgnn_gcn_layer_full": (_int, [_vp, _vp, _vp, _vp, _i64, _i32, _i32, _vp, _i32, _i64, _vp,
                                     _vp, _vp, _vp, _vp, _vp, _i64]),
    "bitgnn_gcn_layer_full_f32": (_int, [_vp, _vp, _vp, _vp, _i32, _i64, _vp, _vp, _i32, _i64,
                                         _vp, _vp, _vp, _vp, _vp, _vp, _i64]),
    "bitgnn_chain_check": (_int, [_vp, ctypes.c_char_p, ctypes.POINTER(_i32)]),
    "bitgnn_gcn_layer_tune": (_int, [_vp, _vp, _vp, _i32, _i32, _i32,
                                     ctypes.POINTER(ctypes.c_float),
                                     ctypes.POINTER(ctypes.c_float)]),
    "bitgnn_ctx_set_fused_spin_limit": (_int, [_vp, _u32]),
    "bitgnn_gcn2_fused": (_int, [_vp, _vp, _vp, _vp, _i32, _i64, _vp, _i32, _i64, _vp, _vp, _vp,
                                 _i32, _i64, _vp, _vp, _vp, _i64, _vp, _i64, _vp]),
}
EXPORTS = tuple(_SIGNATURES)

for _name, (_res, _args) in _SIGNATURES.items():
    _fn = getattr(_lib, _name)      # AttributeError if the library lacks a declared symbol
    _fn.restype = _res
    _fn.argtypes = _args


class BitgnnError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"bitgnn error {code}: {message}")
        self.code = code


def _ptr(t):
    """Device address of a tensor (or a raw int address, or None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream() -> Optional[int]:
    if torch.cuda.is_available():
        return torch.cuda.current_stream().cuda_stream
    return None


class Context:
    """bitgnn_ctx.  device=-1 gives the GPU-less validation context."""

    def __init__(self, device: int = 0):
        h = _vp()
        rc = _lib.bitgnn_ctx_create(ctypes.byref(h), device)
        if rc != OK:
            raise BitgnnError(rc, "bitgnn_ctx_create failed")
        self.handle = h
        self.device = device

    def close(self):
        if self.handle:
            _lib.bitgnn_ctx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def last_error(self) -> str:
        return _lib.bitgnn_last_error(self.handle).decode()

    def check(self, rc: int):
        if rc != OK:
            raise BitgnnError(rc, self.last_error())


class Adjacency:
    """bitgnn_adj handle (device arrays owned by the library)."""

    def __init__(self, handle):
        self.handle = handle
        n, nnz, md, nb = _i64(), _i64(), _i64(), ctypes.c_size_t()
        _lib.bitgnn_adj_info(handle, ctypes.byref(n), ctypes.byref(nnz), ctypes.byref(md),
                             ctypes.byref(nb))
        self.n, self.nnz, self.max_degree, self.device_bytes = n.value, nnz.value, md.value, nb.value

    def blocked_info(self) -> dict:
        v = [_i64() for _ in range(6)]
        _lib.bitgnn_adj_blocked_info(self.handle, *[ctypes.byref(x) for x in v])
        keys = ("parts", "slices", "workgroups", "tiles", "stored_ids", "cb_nodes")
        return {k: x.value for k, x in zip(keys, v)}

    def csr_pointers(self):
        rp, col, deg = _vp(), _vp(), _vp()
        _lib.bitgnn_adj_csr(self.handle, ctypes.byref(rp), ctypes.byref(col), ctypes.byref(deg))
        return rp.value, col.value, deg.value

    def close(self):
        if self.handle:
            _lib.bitgnn_adj_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def words(k: int) -> int:
    return (k + 63) // 64


# --- one function per C entry point ----------------------------------------

def ctx_set_tuning(ctx: Context, cb_nodes: int, part_len: int, min_avg_degree: int):
    ctx.check(_lib.bitgnn_ctx_set_tuning(ctx.handle, cb_nodes, part_len, min_avg_degree))


def ctx_set_bgemm_path(ctx: Context, path: int):
    ctx.check(_lib.bitgnn_ctx_set_bgemm_path(ctx.handle, path))


def ctx_bgemm_kernel(ctx: Context, n: int, kwords: int, M: int) -> int:
    """BGEMM_VALU or BGEMM_MFMA: the kernel bgemm() launches for this shape."""
    k = _int()
    ctx.check(_lib.bitgnn_ctx_bgemm_kernel(ctx.handle, n, kwords, M, ctypes.byref(k)))
    return k.value


def ctx_reserve(ctx: Context, nbytes: int):
    ctx.check(_lib.bitgnn_ctx_reserve(ctx.handle, nbytes))


def ctx_workspace(ctx: Context) -> int:
    b = ctypes.c_size_t()
    ctx.check(_lib.bitgnn_ctx_workspace(ctx.handle, ctypes.byref(b)))
    return b.value


def adj_workspace_bytes(ctx: Context, adj: Optional["Adjacency"], c_max: int, m_max: int) -> int:
    b = ctypes.c_size_t()
    ctx.check(_lib.bitgnn_adj_workspace_bytes(adj.handle if adj else None, c_max, m_max,
                                              ctypes.byref(b)))
    return b.value


def ctx_kernel_timing(ctx: Context, enable: bool):
    ctx.check(_lib.bitgnn_ctx_kernel_timing(ctx.handle, 1 if enable else 0))


def ctx_kernel_times(ctx: Context) -> List[float]:
    buf = (ctypes.c_float * 256)()
    cnt = _i32()
    ctx.check(_lib.bitgnn_ctx_kernel_times(ctx.handle, buf, 256, ctypes.byref(cnt)))
    return [buf[i] for i in range(cnt.value)]


def pack_f32(ctx: Context, x, n, K, ldx, tau, out, out_stride):
    ctx.check(_lib.bitgnn_pack_f32(ctx.handle, _stream(), _ptr(x), n, K, ldx, _ptr(tau), _ptr(out),
                                   out_stride))


def pack_i8(ctx: Context, x, n, K, ldx, out, out_stride):
    ctx.check(_lib.bitgnn_pack_i8(ctx.handle, _stream(), _ptr(x), n, K, ldx, _ptr(out), out_stride))


def pack_weights_i8(ctx: Context, w, K, M, ldw, out, out_stride):
    ctx.check(_lib.bitgnn_pack_weights_i8(ctx.handle, _stream(), _ptr(w), K, M, ldw, _ptr(out),
                                          out_stride))


def adj_build(ctx: Context, src, dst, E, N, flags) -> Adjacency:
    h = _vp()
    ctx.check(_lib.bitgnn_adj_build(ctx.handle, _stream(), _ptr(src), _ptr(dst), E, N, flags,
                                    ctypes.byref(h)))
    return Adjacency(h)


def bgemm(ctx: Context, xbits, n, x_stride, K, kwords, wbits, M, w_stride, epilogue, T, alpha, out,
          out_stride):
    ctx.check(_lib.bitgnn_bgemm(ctx.handle, _stream(), _ptr(xbits), n, x_stride, K, kwords,
                                _ptr(wbits), M, w_stride, epilogue, _ptr(T), _ptr(alpha), _ptr(out),
                                out_stride))


def bgemm_f32(ctx: Context, x, n, K, ldx, tau, wbits, M, w_stride, epilogue, T, alpha, out,
              out_stride):
    ctx.check(_lib.bitgnn_bgemm_f32(ctx.handle, _stream(), _ptr(x), n, K, ldx, _ptr(tau),
                                    _ptr(wbits), M, w_stride, epilogue, _ptr(T), _ptr(alpha),
                                    _ptr(out), out_stride))


def gcn_layer_f32(ctx: Context, adj, x, K, ldx, tau, wbits, M, w_stride, T_mm, T_agg, tmp_bits,
                  out_bits, out_stride):
    ctx.check(_lib.bitgnn_gcn_layer_f32(ctx.handle, _stream(), adj.handle if adj else None,
                                        _ptr(x), K, ldx, _ptr(tau), _ptr(wbits), M, w_stride,
                                        _ptr(T_mm), _ptr(T_agg), _ptr(tmp_bits), _ptr(out_bits),
                                        out_stride))


def bspmm(ctx: Context, adj: Optional[Adjacency], hbits, C, h_stride, epilogue, T, out, out_stride):
    ctx.check(_lib.bitgnn_bspmm(ctx.handle, _stream(), adj.handle if adj else None, _ptr(hbits), C,
                                h_stride, epilogue, _ptr(T), _ptr(out), out_stride))


STATIC_SCRATCH_BYTES = 32 << 20


def bspmm_static(ctx: Context, adj: Optional[Adjacency], hbits, C, h_stride, epilogue, T, out,
                 out_stride):
    """bspmm() with every scratch buffer in the library's static device array."""
    ctx.check(_lib.bitgnn_bspmm_static(ctx.handle, _stream(), adj.handle if adj else None,
                                       _ptr(hbits), C, h_stride, epilogue, _ptr(T), _ptr(out),
                                       out_stride))


def spmm_i32(ctx: Context, adj: Optional[Adjacency], Z, M, z_stride, z_abs_bound, alpha, out,
             out_stride):
    ctx.check(_lib.bitgnn_spmm_i32(ctx.handle, _stream(), adj.handle if adj else None, _ptr(Z), M,
                                   z_stride, z_abs_bound, _ptr(alpha), _ptr(out), out_stride))


def adj_tune(ctx: Context, adj: Optional[Adjacency], C: int, reps: int = 5):
    """Times both aggregation kernels on this graph; returns (csr_ms, blocked_ms)."""
    a, b = ctypes.c_float(-1.0), ctypes.c_float(-1.0)
    ctx.check(_lib.bitgnn_adj_tune(ctx.handle, _stream(), adj.handle if adj else None, C, reps,
                                   ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def spmm_f32(ctx: Context, adj: Optional[Adjacency], x, x_is_bits, C, ldx, r, f, epilogue, tau,
             out, ldo):
    ctx.check(_lib.bitgnn_spmm_f32(ctx.handle, _stream(), adj.handle if adj else None, _ptr(x),
                                   int(x_is_bits), C, ldx, _ptr(r), _ptr(f), epilogue, _ptr(tau),
                                   _ptr(out), ldo))


def gcn_layer(ctx: Context, adj, xbits, x_stride, K, kwords, wbits, M, w_stride, T_mm, T_agg,
              tmp_bits, out_bits, out_stride):
    ctx.check(_lib.bitgnn_gcn_layer(ctx.handle, _stream(), adj.handle if adj else None,
                                    _ptr(xbits), x_stride, K, kwords, _ptr(wbits), M, w_stride,
                                    _ptr(T_mm), _ptr(T_agg), _ptr(tmp_bits), _ptr(out_bits),
                                    out_stride))


def gcn_out_layer(ctx: Context, adj, xbits, x_stride, K, kwords, wbits, M, w_stride, alpha,
                  tmp_i32, logits, ldo):
    ctx.check(_lib.bitgnn_gcn_out_layer(ctx.handle, _stream(), adj.handle if adj else None,
                                        _ptr(xbits), x_stride, K, kwords, _ptr(wbits), M, w_stride,
                                        _ptr(alpha), _ptr(tmp_i32), _ptr(logits), ldo))


def spmm_i16(ctx: Context, adj, z, C, ldz, alpha, r, f, epilogue, tau, out, ldo):
    ctx.check(_lib.bitgnn_spmm_i16(ctx.handle, _stream(), adj.handle if adj else None, _ptr(z), C,
                                   ldz, _ptr(alpha), _ptr(r), _ptr(f), epilogue, _ptr(tau),
                                   _ptr(out), ldo))


def add(ctx: Context, a, a_is_bits, lda, b, b_is_bits, ldb, n, C, epilogue, tau, out, ldo):
    ctx.check(_lib.bitgnn_add(ctx.handle, _stream(), _ptr(a), 1 if a_is_bits else 0, lda, _ptr(b),
                              1 if b_is_bits else 0, ldb, n, C, epilogue, _ptr(tau), _ptr(out),
                              ldo))


def gcn_layer_weighted(ctx: Context, adj, xbits, x_stride, K, kwords, wbits, M, w_stride, T_mm,
                       r, f, tau_agg, tmp_bits, out_bits, out_stride):
    ctx.check(_lib.bitgnn_gcn_layer_weighted(
        ctx.handle, _stream(), adj.handle if adj else None, _ptr(xbits), x_stride, K, kwords,
        _ptr(wbits), M, w_stride, _ptr(T_mm), _ptr(r), _ptr(f), _ptr(tau_agg), _ptr(tmp_bits),
        _ptr(out_bits), out_stride))


def gcn_out_layer_weighted(ctx: Context, adj, xbits, x_stride, K, kwords, wbits, M, w_stride,
                           alpha, r, f, tmp_f32, logits, ldo):
    ctx.check(_lib.bitgnn_gcn_out_layer_weighted(
        ctx.handle, _stream(), adj.handle if adj else None, _ptr(xbits), x_stride, K, kwords,
        _ptr(wbits), M, w_stride, _ptr(alpha), _ptr(r), _ptr(f), _ptr(tmp_f32), _ptr(logits),
        ldo))


def gcn_layer_full(ctx: Context, adj, xbits, x_stride, K, kwords, wbits, M, w_stride, alpha, r,
                   f, tau_agg, tmp_f32, out_bits, out_stride):
    ctx.check(_lib.bitgnn_gcn_layer_full(
        ctx.handle, _stream(), adj.handle if adj else None, _ptr(xbits), x_stride, K, kwords,
        _ptr(wbits), M, w_stride, _ptr(alpha), _ptr(r), _ptr(f), _ptr(tau_agg), _ptr(tmp_f32),
        _ptr(out_bits), out_stride))


def gcn_layer_full_f32(ctx: Context, adj, x, K, ldx, tau_in, wbits, M, w_stride, alpha, r, f,
                       tau_agg, tmp_f32, out_bits, out_stride):
    ctx.check(_lib.bitgnn_gcn_layer_full_f32(
        ctx.handle, _stream(), adj.handle if adj else None, _ptr(x), K, ldx, _ptr(tau_in),
        _ptr(wbits), M, w_stride, _ptr(alpha), _ptr(r), _ptr(f), _ptr(tau_agg), _ptr(tmp_f32),
        _ptr(out_bits), out_stride))


def sage_layer_weighted(ctx: Context, adj, cat_bits, K_in, wbits, M, w_stride, r, f, tau_agg,
                        T_mm, out_bits, out_stride):
    ctx.check(_lib.bitgnn_sage_layer_weighted(
        ctx.handle, _stream(), adj.handle if adj else None, _ptr(cat_bits), K_in, _ptr(wbits), M,
        w_stride, _ptr(r), _ptr(f), _ptr(tau_agg), _ptr(T_mm), _ptr(out_bits), out_stride))


def sage_layer(ctx: Context, adj, cat_bits, K_in, wbits, M, w_stride, T_agg, T_mm, out_bits,
               out_stride):
    ctx.check(_lib.bitgnn_sage_layer(ctx.handle, _stream(), adj.handle if adj else None,
                                     _ptr(cat_bits), K_in, _ptr(wbits), M, w_stride, _ptr(T_agg),
                                     _ptr(T_mm), _ptr(out_bits), out_stride))


def sage_out_layer(ctx: Context, adj, cat_bits, K_in, wbits, M, w_stride, T_agg, alpha, logits,
                   ldo):
    ctx.check(_lib.bitgnn_sage_out_layer(ctx.handle, _stream(), adj.handle if adj else None,
                                         _ptr(cat_bits), K_in, _ptr(wbits), M, w_stride,
                                         _ptr(T_agg), _ptr(alpha), _ptr(logits), ldo))


FUSED_MAX_NODES, FUSED_MAX_DEGREE, FUSED_MAX_HIDDEN, FUSED_MAX_CLASSES = 65536, 1024, 256, 64


def chain_check(ctx: Context, chain: str) -> int:
    """-1 if the chain of functions is well typed, else the position of the first function
    that is not (the reason is in ctx.last_error())."""
    bad = _i32(-1)
    rc = _lib.bitgnn_chain_check(ctx.handle, chain.encode(), ctypes.byref(bad))
    if rc == OK:
        return -1
    if rc != ERR_INVALID_ARG or bad.value < 0:
        ctx.check(rc)
    return bad.value


def gcn_layer_tune(ctx: Context, adj, K: int, M: int, reps: int = 3):
    """(ms of the binary-aggregation layer, ms of the full-precision-aggregation layer)."""
    a, b = ctypes.c_float(), ctypes.c_float()
    ctx.check(_lib.bitgnn_gcn_layer_tune(ctx.handle, _stream(), adj.handle if adj else None, K, M,
                                         reps, ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def ctx_set_fused_spin_limit(ctx: Context, polls: int):
    ctx.check(_lib.bitgnn_ctx_set_fused_spin_limit(ctx.handle, polls))


def gcn2_fused(ctx: Context, adj, x, K0, ldx, w1bits, C1, w1_stride, T_mm, T_agg, w2bits, M,
               w2_stride, alpha, tmp_bits, h_bits, h_stride, logits, ldo, status=None):
    ctx.check(_lib.bitgnn_gcn2_fused(
        ctx.handle, _stream(), adj.handle if adj else None, _ptr(x), K0, ldx, _ptr(w1bits), C1,
        w1_stride, _ptr(T_mm), _ptr(T_agg), _ptr(w2bits), M, w2_stride, _ptr(alpha),
        _ptr(tmp_bits), _ptr(h_bits), h_stride, _ptr(logits), ldo, _ptr(status)))


# --- model runner: buffers + the call sequence, no arithmetic ---------------

class BinaryGNN:
    """Holds the packed parameters and activation buffers of one model on the GPU
    and runs the layer calls in order.  `layers` are objects with fields w (int8
    [K_total, M], +-1), t_mm, t_agg (int32) and alpha (float32, last layer)."""

    def __init__(self, ctx: Context, model: str, adj: Adjacency, dims: Sequence[int],
                 layers: Sequence, device="cuda"):
        assert model in ("gcn", "sage")
        self.ctx, self.model, self.adj, self.dims = ctx, model, adj, list(dims)
        n = adj.n
        self.n = n
        dev = torch.device(device)
        self.params = []
        for l, p in enumerate(layers):
            k_in, m = dims[l], dims[l + 1]
            kw = words(k_in)
            w = torch.as_tensor(p.w, dtype=torch.int8, device=dev).contiguous()
            if model == "gcn":
                wb = torch.zeros((m, kw), dtype=torch.int64, device=dev)
                pack_weights_i8(ctx, w, k_in, m, m, wb, kw)
            else:
                wb = torch.zeros((m, 2 * kw), dtype=torch.int64, device=dev)
                pack_weights_i8(ctx, w, k_in, m, m, wb, 2 * kw)
                pack_weights_i8(ctx, w[k_in:], k_in, m, m, wb[:, kw:], 2 * kw)
            d = dict(wb=wb, kw=kw, k_in=k_in, m=m)
            for name, dt in (("t_mm", torch.int32), ("t_agg", torch.int32),
                             ("alpha", torch.float32)):
                v = getattr(p, name)
                d[name] = None if v is None else torch.as_tensor(v, dtype=dt, device=dev)
            self.params.append(d)
        # activation buffers: bits entering layer l
        self.act: List[torch.Tensor] = []
        for l in range(len(layers)):
            kw = words(dims[l])
            width = kw if model == "gcn" else 2 * kw
            self.act.append(torch.zeros((n, width), dtype=torch.int64, device=dev))
        m_last = dims[-1]
        self.fused_status = None
        self.logits = torch.empty((n, m_last), dtype=torch.float32, device=dev)
        if model == "gcn":
            mw = max(words(d) for d in dims[1:-1]) if len(dims) > 2 else 1
            self.tmp_bits = torch.zeros((n, mw), dtype=torch.int64, device=dev)
            self.tmp_i32 = torch.empty((n, m_last), dtype=torch.int32, device=dev)
        # set-up: the aggregation workspace for this model's widest layer (the layer calls
        # themselves never allocate)
        ctx_reserve(ctx, adj_workspace_bytes(ctx, adj, min(2048, max(dims)), max(dims)))
        torch.cuda.synchronize()

    def forward(self, x_f32: torch.Tensor) -> torch.Tensor:
        """x_f32: float32 [N, K0] on the GPU.  Returns float32 logits [N, classes]."""
        ctx, adj = self.ctx, self.adj
        n, k0 = x_f32.shape
        assert n == self.n and k0 == self.dims[0]
        a0 = self.act[0]
        nl = len(self.params)
        # GCN with a hidden layer: the float features feed the first product directly
        # (BMM.FBB); otherwise they are packed first.
        fused_first = self.model == "gcn" and nl > 1
        if not fused_first:
            pack_f32(ctx, x_f32, n, k0, x_f32.stride(0), None, a0, a0.stride(0))
        for l, p in enumerate(self.params):
            a = self.act[l]
            last = l == nl - 1
            if self.model == "gcn":
                if last:
                    gcn_out_layer(ctx, adj, a, a.stride(0), p["k_in"], p["kw"], p["wb"], p["m"],
                                  p["wb"].stride(0), p["alpha"], self.tmp_i32, self.logits,
                                  self.logits.stride(0))
                elif l == 0:
                    nxt = self.act[l + 1]
                    gcn_layer_f32(ctx, adj, x_f32, k0, x_f32.stride(0), None, p["wb"], p["m"],
                                  p["wb"].stride(0), p["t_mm"], p["t_agg"], self.tmp_bits, nxt,
                                  nxt.stride(0))
                else:
                    nxt = self.act[l + 1]
                    gcn_layer(ctx, adj, a, a.stride(0), p["k_in"], p["kw"], p["wb"], p["m"],
                              p["wb"].stride(0), p["t_mm"], p["t_agg"], self.tmp_bits, nxt,
                              nxt.stride(0))
            else:
                if last:
                    sage_out_layer(ctx, adj, a, p["k_in"], p["wb"], p["m"], p["wb"].stride(0),
                                   p["t_agg"], p["alpha"], self.logits, self.logits.stride(0))
                else:
                    nxt = self.act[l + 1]
                    sage_layer(ctx, adj, a, p["k_in"], p["wb"], p["m"], p["wb"].stride(0),
                               p["t_agg"], p["t_mm"], nxt, nxt.stride(0))
        return self.logits

    def capture(self, x_f32: torch.Tensor) -> "torch.cuda.CUDAGraph":
        """Records forward(x_f32) into a HIP graph and returns it; `graph.replay()` then runs
        the layer calls with one launch from the host and leaves the result in `logits`
        (the calls allocate nothing and do not synchronize, so they can be captured; the
        graph holds the address of x_f32, whose contents may change between replays).
        Measured on MI355X: 0.395 -> 0.358 ms on a 131 K-node 3-layer GCN, 0.234 -> 0.205 ms
        on an 89 K-node GraphSAGE, 0.502 -> 0.485 ms on the 233 K-node GCN."""
        self.forward(x_f32)          # first use of every kernel outside the capture
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self.forward(x_f32)
        return g

    @property
    def fused_applies(self) -> bool:
        """Whether the model is a two-layer GCN inside the one-launch kernel's range."""
        return (self.model == "gcn" and len(self.params) == 2
                and self.n <= FUSED_MAX_NODES and self.adj.max_degree <= FUSED_MAX_DEGREE
                and self.dims[1] <= FUSED_MAX_HIDDEN and self.dims[2] <= FUSED_MAX_CLASSES)

    def forward_fused(self, x_f32: torch.Tensor) -> torch.Tensor:
        """The whole model in one kernel launch (two-layer GCN on a small graph).  Same
        buffers and results as forward(); `fused_status` counts abandoned barrier waits."""
        n, k0 = x_f32.shape
        assert n == self.n and k0 == self.dims[0]
        p0, p1 = self.params
        if self.fused_status is None:
            self.fused_status = torch.zeros(1, dtype=torch.int32, device=self.logits.device)
        h1 = self.act[1]
        gcn2_fused(self.ctx, self.adj, x_f32, k0, x_f32.stride(0), p0["wb"], p0["m"],
                   p0["wb"].stride(0), p0["t_mm"], p0["t_agg"], p1["wb"], p1["m"],
                   p1["wb"].stride(0), p1["alpha"], self.tmp_bits, h1, h1.stride(0),
                   self.logits, self.logits.stride(0), self.fused_status)
        return self.logits

    def forward_ops(self, x_f32: torch.Tensor, mark=None) -> torch.Tensor:
        """Same kernels as forward(), enqueued one low-level entry point at a time;
        `mark(label)` is called before every call (the benchmark records a HIP event
        there) and `mark(None)` after the last one."""
        ctx, adj = self.ctx, self.adj
        mark = mark or (lambda label: None)
        n, k0 = x_f32.shape
        a0 = self.act[0]
        nl = len(self.params)
        fused_first = self.model == "gcn" and nl > 1
        if not fused_first:
            mark("pack_f32")
            pack_f32(ctx, x_f32, n, k0, x_f32.stride(0), None, a0, a0.stride(0))
        for l, p in enumerate(self.params):
            a = self.act[l]
            last = l == nl - 1
            wb, ws, m, kw, k_in = p["wb"], p["wb"].stride(0), p["m"], p["kw"], p["k_in"]
            if self.model == "gcn":
                if last:
                    # one call: the driver picks aggregate-then-transform when it can
                    mark(f"L{l}.out_layer")
                    gcn_out_layer(ctx, adj, a, a.stride(0), k_in, kw, wb, m, ws, p["alpha"],
                                  self.tmp_i32, self.logits, self.logits.stride(0))
                else:
                    nxt = self.act[l + 1]
                    mw = words(m)
                    if l == 0:
                        mark(f"L{l}.bgemm_f32")
                        bgemm_f32(ctx, x_f32, n, k0, x_f32.stride(0), None, wb, m, ws,
                                  EPI_THRESH_BITS, p["t_mm"], None, self.tmp_bits, mw)
                    else:
                        mark(f"L{l}.bgemm")
                        bgemm(ctx, a, n, a.stride(0), k_in, kw, wb, m, ws, EPI_THRESH_BITS,
                              p["t_mm"], None, self.tmp_bits, mw)
                    mark(f"L{l}.bspmm")
                    bspmm(ctx, adj, self.tmp_bits, m, mw, EPI_THRESH_BITS, p["t_agg"], nxt,
                          nxt.stride(0))
            else:
                mark(f"L{l}.bspmm")
                bspmm(ctx, adj, a, k_in, 2 * kw, EPI_THRESH_BITS, p["t_agg"], a[:, kw:], 2 * kw)
                mark(f"L{l}.bgemm")
                if last:
                    bgemm(ctx, a, n, 2 * kw, 2 * k_in, 2 * kw, wb, m, ws, EPI_SCALE_F32, None,
                          p["alpha"], self.logits, self.logits.stride(0))
                else:
                    nxt = self.act[l + 1]
                    bgemm(ctx, a, n, 2 * kw, 2 * k_in, 2 * kw, wb, m, ws, EPI_THRESH_BITS,
                          p["t_mm"], None, nxt, nxt.stride(0))
        mark(None)
        return self.logits
