"""Python face of the CPU oracle (TEST INFRASTRUCTURE ONLY).

The arithmetic lives in `bitgnn_oracle.c` (plain loops on unpacked +-1 int8
arrays, int64 accumulators).  This file compiles and loads it, builds the
adjacency as a *set* of pairs with numpy, chains the per-step functions into the
layer recipes of the paper, and holds a deliberately trivial bit packer used
only to compare against the library's packed words.

Nothing here imports or calls the HIP library, and the library never imports
this module.  Only tests, the smoke check and the benchmark's cpu_baseline leg
use it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bitgnn_oracle.c")
_LIB = os.path.join(_HERE, "libbitgnn_oracle.so")

ADJ_SYMMETRIZE = 1
ADJ_ADD_SELF_LOOPS = 2


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc -O2 -fopenmp (no -march: the binary must
    run on whatever host the GPU machine has)."""
    if force or not os.path.exists(_LIB) or \
            os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
                               "-std=c99", "-Wall", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_max_threads.restype = ctypes.c_int
    return _lib


def max_threads() -> int:
    return int(lib().orc_max_threads())


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


I64 = ctypes.c_int64


# ---------------------------------------------------------------------------
# per-step functions
# ---------------------------------------------------------------------------

def bin_f32(x: np.ndarray, tau: Optional[np.ndarray] = None) -> np.ndarray:
    """Section 2.2 sign rule: +1 where x >= tau (tau = 0 if None), else -1."""
    x = _c(x, np.float32)
    n, k = x.shape
    v = np.empty((n, k), dtype=np.int8)
    tau_c = None if tau is None else _c(tau, np.float32)
    lib().orc_bin_f32(_p(x), I64(n), I64(k), I64(k), _p(tau_c), _p(v))
    return v


def bin_i8(x: np.ndarray) -> np.ndarray:
    x = _c(x, np.int8)
    n, k = x.shape
    v = np.empty((n, k), dtype=np.int8)
    lib().orc_bin_i8(_p(x), I64(n), I64(k), I64(k), _p(v))
    return v


def adjacency(src: np.ndarray, dst: np.ndarray, n: int, flags: int
              ) -> Tuple[np.ndarray, np.ndarray]:
    """A_hat as a set of (row, col) pairs (Section 2.1: A_hat = A + I when self
    loops are asked for; duplicates collapse; SYMMETRIZE adds every reversed
    pair).  Returns CSR (rowptr int64 [n+1], col int32 [nnz]); row i lists
    N(i) = { j : A_hat[i][j] = 1 } in increasing j."""
    s = np.asarray(src, dtype=np.int64)
    d = np.asarray(dst, dtype=np.int64)
    if len(s) and (s.min() < 0 or d.min() < 0 or s.max() >= n or d.max() >= n):
        raise ValueError("edge endpoint out of range")
    keys = [s * n + d]
    if flags & ADJ_SYMMETRIZE:
        keys.append(d * n + s)
    if flags & ADJ_ADD_SELF_LOOPS:
        i = np.arange(n, dtype=np.int64)
        keys.append(i * n + i)
    key = np.unique(np.concatenate(keys))
    row = key // n
    col = (key - row * n).astype(np.int32)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(row, minlength=n), out=rowptr[1:])
    return rowptr, col


def degrees(rowptr: np.ndarray) -> np.ndarray:
    return np.diff(rowptr).astype(np.int64)


def bmm(vx: np.ndarray, vw: np.ndarray) -> np.ndarray:
    """Z = vx @ vw on +-1 int8 operands by the literal triple loop."""
    vx = _c(vx, np.int8)
    vw = _c(vw, np.int8)
    n, k = vx.shape
    k2, m = vw.shape
    assert k == k2
    z = np.empty((n, m), dtype=np.int64)
    lib().orc_bmm(_p(vx), I64(n), I64(k), _p(vw), I64(m), _p(z))
    return z


def spmm_pm1(rowptr: np.ndarray, col: np.ndarray, v: np.ndarray,
             rows: Optional[Tuple[int, int]] = None) -> np.ndarray:
    """S[i] = sum of the +-1 rows v[j], j in N(i) (if/else walk, method 1).
    `rows=(lo, hi)` restricts the output to rows lo..hi-1."""
    v = _c(v, np.int8)
    rowptr = _c(rowptr, np.int64)
    col = _c(col, np.int32)
    lo, hi = (0, len(rowptr) - 1) if rows is None else rows
    c = v.shape[1]
    s = np.empty((hi - lo, c), dtype=np.int64)
    rp = rowptr[lo:hi + 1]
    lib().orc_spmm_pm1(_p(rp), _p(col), I64(hi - lo), _p(v), I64(c), _p(s))
    return s


def rebin(acc: np.ndarray, t: np.ndarray) -> np.ndarray:
    """+1 where acc >= T_c else -1."""
    acc = _c(acc, np.int64)
    t = _c(t, np.int32)
    n, c = acc.shape
    assert t.shape == (c,)
    v = np.empty((n, c), dtype=np.int8)
    lib().orc_rebin(_p(acc), I64(n), I64(c), _p(t), _p(v))
    return v


def spmm_i64(rowptr: np.ndarray, col: np.ndarray, z: np.ndarray,
             rows: Optional[Tuple[int, int]] = None) -> np.ndarray:
    """Y[i] = sum of the integer rows Z[j], j in N(i)."""
    z = _c(z, np.int64)
    rowptr = _c(rowptr, np.int64)
    col = _c(col, np.int32)
    lo, hi = (0, len(rowptr) - 1) if rows is None else rows
    m = z.shape[1]
    y = np.empty((hi - lo, m), dtype=np.int64)
    rp = rowptr[lo:hi + 1]
    lib().orc_spmm_i64(_p(rp), _p(col), I64(hi - lo), _p(z), I64(m), _p(y))
    return y


def spmm_weighted(rowptr: np.ndarray, col: np.ndarray, x: np.ndarray,
                  r: Optional[np.ndarray] = None, f: Optional[np.ndarray] = None) -> np.ndarray:
    """Y[i] = r_i * sum_{j in N(i)} f_j x[j] in float64: the plain definition of the
    weighted / full-precision aggregation (Section 3.1.1).  x: any real [n, C]."""
    x = _c(x, np.float64)
    rowptr = _c(rowptr, np.int64)
    col = _c(col, np.int32)
    n, c = len(rowptr) - 1, x.shape[1]
    r = None if r is None else _c(r, np.float64)
    f = None if f is None else _c(f, np.float64)
    y = np.empty((n, c), dtype=np.float64)
    lib().orc_spmm_weighted(_p(rowptr), _p(col), I64(n), _p(x), I64(c), _p(r), _p(f), _p(y))
    return y


def spmm_weighted_f32(rowptr: np.ndarray, col: np.ndarray, x: np.ndarray,
                      r: Optional[np.ndarray] = None, f: Optional[np.ndarray] = None,
                      rows: Optional[Tuple[int, int]] = None) -> np.ndarray:
    """The same sum in float32, every step rounded once, neighbours in stored order:
    the value that decides a bit when the result is binarized again."""
    x = _c(x, np.float32)
    rowptr = _c(rowptr, np.int64)
    col = _c(col, np.int32)
    lo, hi = (0, len(rowptr) - 1) if rows is None else rows
    c = x.shape[1]
    r = None if r is None else _c(np.asarray(r, dtype=np.float32)[lo:hi], np.float32)
    f = None if f is None else _c(f, np.float32)
    y = np.empty((hi - lo, c), dtype=np.float32)
    rp = rowptr[lo:hi + 1]
    lib().orc_spmm_weighted_f32(_p(rp), _p(col), I64(hi - lo), _p(x), I64(c), _p(r), _p(f),
                                _p(y))
    return y


def rebin_f32(y: np.ndarray, tau: np.ndarray) -> np.ndarray:
    """+1 where y >= tau_c else -1, on float32 values."""
    y = _c(y, np.float32)
    tau = _c(tau, np.float32)
    n, c = y.shape
    assert tau.shape == (c,)
    v = np.empty((n, c), dtype=np.int8)
    lib().orc_rebin_f32(_p(y), I64(n), I64(c), _p(tau), _p(v))
    return v


def add_f32(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """ADD, the auxiliary merge of two activation tensors (Section 3.1.2, ADD.BBF /
    ADD.FFF): element-wise a + b in float32 (the paper's full precision), one rounded
    addition.  Operands are float32 arrays or +-1 int8 arrays (binary tensors)."""
    assert a.shape == b.shape and a.ndim == 2
    fa = np.ascontiguousarray(a, dtype=np.float32)
    fb = np.ascontiguousarray(b, dtype=np.float32)
    return np.add(fa, fb, dtype=np.float32)


def sage_hidden_layer_added(rowptr, col, v, w_self, w_nb, t_agg, t_mm) -> np.ndarray:
    """GraphSAGE hidden layer with the self-connectivity merged by addition (Section 2.1:
    X_i W1 + aggregate(X_j) W2; Section 3.1.2: the merge is an ADD of the two products),
    in exact integers: bin(bmm(v, W1) + bmm(bin(A v), W2))."""
    nb = _spmm_rebin(rowptr, col, v, t_agg)
    return rebin(bmm(v, w_self) + bmm(nb, w_nb), t_mm)


def scale(y: np.ndarray, alpha: np.ndarray) -> np.ndarray:
    y = _c(y, np.int64)
    alpha = _c(alpha, np.float32)
    n, m = y.shape
    out = np.empty((n, m), dtype=np.float32)
    lib().orc_scale(_p(y), I64(n), I64(m), _p(alpha), _p(out))
    return out


def concat(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    a = _c(a, np.int8)
    b = _c(b, np.int8)
    n, ka = a.shape
    kb = b.shape[1]
    out = np.empty((n, ka + kb), dtype=np.int8)
    lib().orc_concat(_p(a), I64(ka), _p(b), I64(kb), I64(n), _p(out))
    return out


# ---------------------------------------------------------------------------
# layers and models (the "binary aggregation" recipe of Table 3's caption:
# hidden layers MM.xBB + BSpMM.BBB, last layer MM.BBF + BSpMM.FBF)
# ---------------------------------------------------------------------------

_CHUNK = 1 << 16


def _bmm_rebin(v: np.ndarray, w: np.ndarray, t: np.ndarray) -> np.ndarray:
    """rebin(bmm(v, w), t) in row chunks (bounds the int64 temporary)."""
    out = np.empty((v.shape[0], w.shape[1]), dtype=np.int8)
    for lo in range(0, v.shape[0], _CHUNK):
        out[lo:lo + _CHUNK] = rebin(bmm(v[lo:lo + _CHUNK], w), t)
    return out


def _spmm_rebin(rowptr, col, v, t) -> np.ndarray:
    n = len(rowptr) - 1
    out = np.empty((n, v.shape[1]), dtype=np.int8)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        out[lo:hi] = rebin(spmm_pm1(rowptr, col, v, (lo, hi)), t)
    return out


def gcn_hidden_layer(rowptr, col, v, w, t_mm, t_agg) -> np.ndarray:
    """h = bin_{t_mm}(v W);  out = bin_{t_agg}(A_hat h)."""
    h = _bmm_rebin(v, w, t_mm)
    return _spmm_rebin(rowptr, col, h, t_agg)


def gcn_hidden_layer_norm(rowptr, col, v, w, t_mm, r, f, tau_agg) -> np.ndarray:
    """h = bin_{t_mm}(v W);  out = bin_{tau}(diag(r) A_hat diag(f) h): the GCN layer with a
    weighted (e.g. symmetrically normalised) adjacency through its factor vectors
    (Section 3.1.1); the weighted sum is taken in float32, step by step."""
    h = _bmm_rebin(v, w, t_mm)
    return rebin_f32(spmm_weighted_f32(rowptr, col, h, r, f), tau_agg)


def gcn_hidden_layer_full(rowptr, col, v, w, alpha, r, f, tau_agg) -> np.ndarray:
    """GCN hidden layer with full-precision aggregation (Table 3's "Ours (full)", the
    aggregation of Bi-GCN-1 in Section 3.1): z = alpha * (v W) in float32 (BMM + SCL), then
    out = bin_{tau}(diag(r) A_hat diag(f) z), the weighted sum in float32, step by step."""
    n = v.shape[0]
    z = np.empty((n, w.shape[1]), dtype=np.float32)
    for lo in range(0, n, _CHUNK):
        z[lo:lo + _CHUNK] = scale(bmm(v[lo:lo + _CHUNK], w), alpha)
    return rebin_f32(spmm_weighted_f32(rowptr, col, z, r, f), tau_agg)


def gcn_out_layer_norm(rowptr, col, v, w, alpha, r, f) -> np.ndarray:
    """Z = v W (integers);  logits = diag(r) A_hat diag(f) (alpha * Z): the output layer with
    a weighted adjacency; BMM.BBF with its scale, then the full-precision weighted
    aggregation (float32, step by step)."""
    n = v.shape[0]
    z = np.empty((n, w.shape[1]), dtype=np.float32)
    for lo in range(0, n, _CHUNK):
        z[lo:lo + _CHUNK] = scale(bmm(v[lo:lo + _CHUNK], w), alpha)
    return spmm_weighted_f32(rowptr, col, z, r, f)


def sage_hidden_layer_mean(rowptr, col, v, w, rmean, tau_agg, t_mm) -> np.ndarray:
    """nb = bin_{tau}(mean_{j in N(i)} v_j) with rmean = 1/deg (the mean aggregator of
    Section 2.1);  out = bin_{t_mm}([v | nb] W)."""
    nb = rebin_f32(spmm_weighted_f32(rowptr, col, v, rmean, None), tau_agg)
    out = np.empty((v.shape[0], w.shape[1]), dtype=np.int8)
    for lo in range(0, v.shape[0], _CHUNK):
        cat = concat(v[lo:lo + _CHUNK], nb[lo:lo + _CHUNK])
        out[lo:lo + _CHUNK] = rebin(bmm(cat, w), t_mm)
    return out


def gcn_out_layer(rowptr, col, v, w, alpha) -> np.ndarray:
    """Z = v W (integers);  Y = A_hat Z;  logits = alpha * Y."""
    n = v.shape[0]
    z = np.empty((n, w.shape[1]), dtype=np.int64)
    for lo in range(0, n, _CHUNK):
        z[lo:lo + _CHUNK] = bmm(v[lo:lo + _CHUNK], w)
    out = np.empty((n, w.shape[1]), dtype=np.float32)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        out[lo:hi] = scale(spmm_i64(rowptr, col, z, (lo, hi)), alpha)
    return out


def sage_hidden_layer(rowptr, col, v, w, t_agg, t_mm) -> np.ndarray:
    """nb = bin_{t_agg}(A v);  out = bin_{t_mm}([v | nb] W)  (GraphConv sum
    form, Section 2.1, with the self and neighbour weight blocks stacked)."""
    nb = _spmm_rebin(rowptr, col, v, t_agg)
    out = np.empty((v.shape[0], w.shape[1]), dtype=np.int8)
    for lo in range(0, v.shape[0], _CHUNK):
        cat = concat(v[lo:lo + _CHUNK], nb[lo:lo + _CHUNK])
        out[lo:lo + _CHUNK] = rebin(bmm(cat, w), t_mm)
    return out


def sage_out_layer(rowptr, col, v, w, t_agg, alpha) -> np.ndarray:
    nb = _spmm_rebin(rowptr, col, v, t_agg)
    out = np.empty((v.shape[0], w.shape[1]), dtype=np.float32)
    for lo in range(0, v.shape[0], _CHUNK):
        cat = concat(v[lo:lo + _CHUNK], nb[lo:lo + _CHUNK])
        out[lo:lo + _CHUNK] = scale(bmm(cat, w), alpha)
    return out


def forward(model: str, rowptr, col, v0: np.ndarray, layers: Sequence,
            return_hidden: bool = False):
    """Whole model on +-1 input v0; `layers` are objects with fields
    w, t_mm, t_agg, alpha (alpha set on the last layer only)."""
    v = v0
    hidden: List[np.ndarray] = []
    for l, p in enumerate(layers):
        last = l == len(layers) - 1
        if model == "gcn":
            v = gcn_out_layer(rowptr, col, v, p.w, p.alpha) if last else \
                gcn_hidden_layer(rowptr, col, v, p.w, p.t_mm, p.t_agg)
        elif model == "sage":
            v = sage_out_layer(rowptr, col, v, p.w, p.t_agg, p.alpha) if last else \
                sage_hidden_layer(rowptr, col, v, p.w, p.t_agg, p.t_mm)
        else:
            raise ValueError(model)
        if not last:
            hidden.append(v)
    return (v, hidden) if return_hidden else v


# ---------------------------------------------------------------------------
# comparison helpers (not part of the method)
# ---------------------------------------------------------------------------

def to_words(v: np.ndarray, wpr: Optional[int] = None) -> np.ndarray:
    """+-1 int8 [n][K] -> uint64 [n][wpr]: bit (k % 64) of word (k // 64) is 1
    iff v[i][k] == +1; unused bits are 0.  One Python-level loop per bit
    column: slow and obvious on purpose."""
    n, k = v.shape
    need = (k + 63) // 64
    wpr = need if wpr is None else wpr
    assert wpr >= need
    out = np.zeros((n, wpr), dtype=np.uint64)
    for kk in range(k):
        out[:, kk // 64] |= (v[:, kk] > 0).astype(np.uint64) << np.uint64(kk % 64)
    return out


def from_words(words: np.ndarray, k: int) -> np.ndarray:
    """Inverse of `to_words` for the first k bits."""
    n = words.shape[0]
    v = np.empty((n, k), dtype=np.int8)
    for kk in range(k):
        bit = (words[:, kk // 64] >> np.uint64(kk % 64)) & np.uint64(1)
        v[:, kk] = np.where(bit == 1, 1, -1)
    return v
