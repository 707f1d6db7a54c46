"""Pins for the CPU oracle: each part of it is checked against something other
than itself - the paper's closed forms (Section 2.2, Section 3.2.2), brute
force on tiny inputs, numpy's int64 matmul as an independent library routine,
invariants, hand-worked fixtures under tests/golden/, and a host emulation of
the paper's Algorithm 1.  All of this runs without a GPU.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2305_02522_amd import workloads as W
from tests import alg1_emulator as alg1

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _bits_of(v):          # +-1 vector -> python int, bit k = (v[k] == +1)
    x = 0
    for k, e in enumerate(v):
        if e > 0:
            x |= 1 << k
    return x


def _popc(x):
    return bin(x).count("1")


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- BIN
def test_bin_sign_rule_ties_and_tau():
    x = np.array([[0.0, -0.0, 1e-30, -1e-30, 3.5, -2.0, np.nan]], dtype=np.float32)
    v = orc.bin_f32(x)
    assert v.tolist() == [[1, 1, 1, -1, 1, -1, -1]]
    tau = np.array([0.5, -1, 0, 0, 3.5, -2.0, 0], dtype=np.float32)
    v = orc.bin_f32(x, tau)
    assert v.tolist() == [[-1, 1, 1, -1, 1, 1, -1]]
    assert orc.bin_i8(np.array([[0, -1, 1, -128, 127]], dtype=np.int8)).tolist() == \
        [[1, -1, 1, -1, 1]]


# ---------------------------------------------------------------- BMM
def test_bmm_golden_pm1_dot():
    for line in open(os.path.join(GOLDEN, "pm1_dot.txt")):
        if line.startswith("#") or not line.strip():
            continue
        a, b, n, pc, c = line.split()
        va = np.array([[1 if ch == "1" else -1 for ch in a]], dtype=np.int8)
        vb = np.array([[1 if ch == "1" else -1 for ch in b]], dtype=np.int8).T
        assert len(a) == int(n)
        assert _popc(int(a, 2) ^ int(b, 2)) == int(pc)
        assert orc.bmm(va, vb)[0, 0] == int(c)


def test_bmm_exhaustive_small_k_vs_xor_popc():
    # all 2^K x 2^K pairs: Z = K - 2 popc(x xor w) = 2 popc(xnor) - K
    for K in (1, 2, 3, 5, 7):
        allv = np.array(list(itertools.product((-1, 1), repeat=K)), dtype=np.int8)
        z = orc.bmm(allv, allv.T.copy())
        ints = [_bits_of(v) for v in allv]
        full = (1 << K) - 1
        for i, xi in enumerate(ints):
            for j, wj in enumerate(ints):
                assert z[i, j] == K - 2 * _popc(xi ^ wj)
                assert z[i, j] == 2 * _popc(~(xi ^ wj) & full) - K


@pytest.mark.parametrize("K", [1, 63, 64, 65, 100, 602, 1433])
def test_bmm_random_vs_identity_and_numpy(K):
    r = _rng(K)
    x = W.pm1(r, (37, K))
    w = W.pm1(r, (K, 11))
    z = orc.bmm(x, w)
    assert np.array_equal(z, x.astype(np.int64) @ w.astype(np.int64))
    for i in (0, 17, 36):
        for c in (0, 5, 10):
            assert z[i, c] == K - 2 * _popc(_bits_of(x[i]) ^ _bits_of(w[:, c]))
    assert np.all((z - K) % 2 == 0) and np.all(np.abs(z) <= K)


def test_bmm_special_cases():
    r = _rng(3)
    x = W.pm1(r, (9, 130))
    z = orc.bmm(x, x.T.copy())
    assert np.all(np.diag(z) == 130)              # x = w  -> K
    z = orc.bmm(x, (-x).T.copy())
    assert np.all(np.diag(z) == -130)             # x = -w -> -K
    # not symmetric in shape: a transposed weight operand must fail this
    w = W.pm1(r, (130, 4))
    assert orc.bmm(x, w).shape == (9, 4)


# ---------------------------------------------------------------- adjacency
def test_adjacency_set_semantics_and_degree_invariants():
    r = _rng(11)
    n = 50
    src, dst = W.random_graph(r, n, 400)
    rp, col = orc.adjacency(src, dst, n, 0)
    pairs = set(zip(src.tolist(), dst.tolist()))
    got = {(i, int(j)) for i in range(n) for j in col[rp[i]:rp[i + 1]]}
    assert got == pairs and rp[-1] == len(pairs)
    for i in range(n):                            # sorted, no duplicates
        assert np.all(np.diff(col[rp[i]:rp[i + 1]]) > 0)
    # symmetrise: in-degree == out-degree, membership symmetric
    rp2, col2 = orc.adjacency(src, dst, n, orc.ADJ_SYMMETRIZE)
    got2 = {(i, int(j)) for i in range(n) for j in col2[rp2[i]:rp2[i + 1]]}
    assert got2 == pairs | {(b, a) for a, b in pairs}
    indeg = np.bincount(col2, minlength=n)
    assert np.array_equal(indeg, orc.degrees(rp2))
    # + I: every degree >= 1, nnz grows by N - existing loops
    rp3, col3 = orc.adjacency(src, dst, n, orc.ADJ_SYMMETRIZE | orc.ADJ_ADD_SELF_LOOPS)
    loops = sum(1 for a, b in got2 if a == b)
    assert rp3[-1] == rp2[-1] + n - loops
    assert orc.degrees(rp3).min() >= 1 and orc.degrees(rp3).sum() == rp3[-1]
    # idempotent under duplicate injection and shuffling
    perm = r.permutation(2 * len(src))
    s2 = np.concatenate([src, src])[perm]
    d2 = np.concatenate([dst, dst])[perm]
    rp4, col4 = orc.adjacency(s2, d2, n, orc.ADJ_SYMMETRIZE | orc.ADJ_ADD_SELF_LOOPS)
    assert np.array_equal(rp3, rp4) and np.array_equal(col3, col4)
    with pytest.raises(ValueError):
        orc.adjacency(np.array([0, n]), np.array([0, 0]), n, 0)


# ---------------------------------------------------------------- bit-SpMM
def test_spmm_golden_trinary():
    for line in open(os.path.join(GOLDEN, "trinary_dot.txt")):
        if line.startswith("#") or not line.strip():
            continue
        a, b, pab, panb, pa, dot = line.split()
        n = len(a)
        ai, bi = int(a, 2), int(b, 2)
        full = (1 << n) - 1
        assert _popc(ai & bi) == int(pab) and _popc(ai & ~bi & full) == int(panb)
        assert _popc(ai) == int(pa)
        # one aggregating row (node 0) whose neighbours are the set bits of a
        nbrs = [j for j, ch in enumerate(a) if ch == "1"]
        rp = np.array([0, len(nbrs)] + [len(nbrs)] * (n - 1), dtype=np.int64)
        col = np.array(nbrs, dtype=np.int32)
        v = np.array([[1 if ch == "1" else -1] for ch in b], dtype=np.int8)
        s = orc.spmm_pm1(rp, col, v)
        assert s[0, 0] == int(dot)
        assert int(pab) - int(panb) == int(dot) == 2 * int(pab) - int(pa)


def test_spmm_bruteforce_all_graphs_n3():
    # every 3x3 0/1 adjacency (512 of them) against a fixed +-1 matrix
    v = np.array([[1, -1, 1, 1], [-1, -1, 1, -1], [1, 1, -1, -1]], dtype=np.int8)
    for code in range(512):
        a = np.array([(code >> b) & 1 for b in range(9)], dtype=np.int64).reshape(3, 3)
        src, dst = np.nonzero(a)
        rp, col = orc.adjacency(src, dst, 3, 0)
        assert np.array_equal(orc.spmm_pm1(rp, col, v), a @ v.astype(np.int64))


def test_spmm_three_trinary_methods_and_dense_matmul():
    r = _rng(5)
    n, c = 64, 70
    src, dst = W.random_graph(r, n, 600)
    rp, col = orc.adjacency(src, dst, n, orc.ADJ_SYMMETRIZE | orc.ADJ_ADD_SELF_LOOPS)
    v = W.pm1(r, (n, c))
    s = orc.spmm_pm1(rp, col, v)
    dense = np.zeros((n, n), dtype=np.int64)
    for i in range(n):
        dense[i, col[rp[i]:rp[i + 1]]] = 1
    assert np.array_equal(s, dense @ v.astype(np.int64))
    deg = orc.degrees(rp)
    for i in (0, 13, 63):
        a = sum(1 << int(j) for j in col[rp[i]:rp[i + 1]])
        for ch in (0, 31, 69):
            b = sum(1 << j for j in range(n) if v[j, ch] > 0)
            full = (1 << n) - 1
            m2 = _popc(a & b) - _popc(a & ~b & full)
            m3 = 2 * _popc(a & b) - _popc(a)
            assert s[i, ch] == m2 == m3
    # invariants
    assert np.all((s - deg[:, None]) % 2 == 0) and np.all(np.abs(s) <= deg[:, None])
    assert np.array_equal(s.sum(axis=0), (deg[:, None] * v).sum(axis=0))  # symmetric A
    assert np.array_equal(orc.spmm_pm1(rp, col, np.ones_like(v)), np.tile(deg[:, None], (1, c)))
    assert np.array_equal(orc.spmm_pm1(rp, col, -np.ones_like(v)), -np.tile(deg[:, None], (1, c)))
    # row-range form returns the same rows
    assert np.array_equal(orc.spmm_pm1(rp, col, v, (10, 33)), s[10:33])


def test_spmm_direction_row_aggregates_columns():
    # directed 2-node graph: only A[0][1] = 1.  Row 0 must receive v[1].
    rp, col = orc.adjacency(np.array([0]), np.array([1]), 2, 0)
    v = np.array([[1, 1], [-1, 1]], dtype=np.int8)
    assert orc.spmm_pm1(rp, col, v).tolist() == [[-1, 1], [0, 0]]
    z = np.array([[5, 7], [11, -3]], dtype=np.int64)
    assert orc.spmm_i64(rp, col, z).tolist() == [[11, -3], [0, 0]]


# ---------------------------------------------------------------- threshold
def test_rebin_threshold_properties():
    r = _rng(8)
    acc = r.integers(-9, 10, size=(40, 6)).astype(np.int64)
    zero = np.zeros(6, dtype=np.int32)
    assert np.array_equal(orc.rebin(acc, zero), np.where(acc >= 0, 1, -1))
    prev = None
    for t in range(-10, 12):
        v = orc.rebin(acc, np.full(6, t, dtype=np.int32))
        if prev is not None:
            assert np.all(v <= prev)              # monotone in T
        prev = v
    assert np.all(orc.rebin(acc, np.full(6, -9, dtype=np.int32)) == 1)
    assert np.all(orc.rebin(acc, np.full(6, 10, dtype=np.int32)) == -1)
    t = np.array([-4, -1, 0, 1, 2, 4], dtype=np.int32)   # per channel, tie -> +1
    assert np.array_equal(orc.rebin(acc, t), np.where(acc >= t[None, :], 1, -1))


def test_words_roundtrip_and_pad_bits():
    r = _rng(2)
    for k in (1, 63, 64, 65, 130):
        v = W.pm1(r, (5, k))
        words = orc.to_words(v)
        assert words.shape == (5, (k + 63) // 64)
        assert np.array_equal(orc.from_words(words, k), v)
        for i in range(5):
            x = sum(int(words[i, w]) << (64 * w) for w in range(words.shape[1]))
            assert x == _bits_of(v[i])            # bit k%64 of word k//64, pad bits 0


# ---------------------------------------------------------------- last layer
def test_last_layer_associativity_and_scale():
    r = _rng(21)
    n, k, m = 80, 33, 5
    src, dst = W.random_graph(r, n, 500)
    rp, col = orc.adjacency(src, dst, n, orc.ADJ_SYMMETRIZE | orc.ADJ_ADD_SELF_LOOPS)
    h = W.pm1(r, (n, k))
    w = W.pm1(r, (k, m))
    y = orc.spmm_i64(rp, col, orc.bmm(h, w))                   # A (H W)
    y2 = orc.spmm_pm1(rp, col, h) @ w.astype(np.int64)         # (A H) W
    assert np.array_equal(y, y2)
    ones = np.ones(m, dtype=np.float32)
    assert np.array_equal(orc.scale(y, ones), y.astype(np.float32))
    alpha = r.uniform(0.5, 1.5, m).astype(np.float32)
    out = orc.gcn_out_layer(rp, col, h, w, alpha)
    assert np.allclose(out, alpha.astype(np.float64) * y, rtol=1e-7, atol=0)


# ---------------------------------------------------------------- whole models
def _parse_rows(s, dtype=np.int64):
    return np.array([[float(t) for t in row.split()] for row in s.split("|")]).astype(dtype)


def test_gcn_golden_tiny_handworked():
    f = {}
    for line in open(os.path.join(GOLDEN, "gcn_tiny.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, rest = line.split(None, 1)
        f[key] = rest.strip()
    n = int(f["n"])
    e = [tuple(map(int, p.split("-"))) for p in f["edges"].split()]
    src = np.array([a for a, _ in e])
    dst = np.array([b for _, b in e])
    rp, col = orc.adjacency(src, dst, n, orc.ADJ_SYMMETRIZE | orc.ADJ_ADD_SELF_LOOPS)
    x = _parse_rows(f["x"], np.int8)
    w1 = _parse_rows(f["w1"], np.int8)
    w2 = _parse_rows(f["w2"], np.int8)
    t_mm = np.array(f["t_mm"].split(), dtype=np.int32)
    t_agg = np.array(f["t_agg"].split(), dtype=np.int32)
    z1 = orc.bmm(x, w1)
    assert np.array_equal(z1, _parse_rows(f["z1"]))
    h = orc.rebin(z1, t_mm)
    assert np.array_equal(h, _parse_rows(f["h"]))
    s = orc.spmm_pm1(rp, col, h)
    assert np.array_equal(s, _parse_rows(f["s"]))
    out1 = orc.rebin(s, t_agg)
    assert np.array_equal(out1, _parse_rows(f["out1"]))
    assert np.array_equal(orc.gcn_hidden_layer(rp, col, x, w1, t_mm, t_agg), out1)
    z2 = orc.bmm(out1, w2)
    assert np.array_equal(z2, _parse_rows(f["z2"]))
    assert np.array_equal(orc.spmm_i64(rp, col, z2), _parse_rows(f["y"]))
    alpha = np.array([float(f["alpha"])], dtype=np.float32)
    logits = orc.gcn_out_layer(rp, col, out1, w2, alpha)
    assert np.array_equal(logits, _parse_rows(f["logits"], np.float32))


def _dense_adj(n, rp, col):
    a = np.zeros((n, n), dtype=np.int64)
    for i in range(n):
        a[i, col[rp[i]:rp[i + 1]]] = 1
    return a


def test_config1_gcn_vs_dense_textbook_evaluation():
    wl = W.make_workload(1)
    rp, col = orc.adjacency(wl.src, wl.dst, wl.n, wl.adj_flags)
    nnz_no_loops = rp[-1] - wl.n
    assert 9000 < nnz_no_loops < 12000            # ~10.5k stored non-zeros + N loops
    a = _dense_adj(wl.n, rp, col)
    assert np.array_equal(a, a.T) and np.all(np.diag(a) == 1)
    logits, hidden = orc.forward("gcn", rp, col, wl.x, wl.layers, return_hidden=True)
    l1, l2 = wl.layers
    x = wl.x.astype(np.int64)
    h = np.where(x @ l1.w.astype(np.int64) >= l1.t_mm[None, :], 1, -1)
    out1 = np.where(a @ h >= l1.t_agg[None, :], 1, -1)
    assert np.array_equal(hidden[0], out1)
    y = a @ (out1 @ l2.w.astype(np.int64))
    ref = l2.alpha.astype(np.float64)[None, :] * y
    assert np.allclose(logits, ref, rtol=1e-6, atol=0)
    assert logits.dtype == np.float32 and logits.shape == (wl.n, 7)


def test_sage_small_vs_two_matmul_form():
    # [self | nbr] [W1; W2] == self W1 + nbr W2 (GraphConv sum form), no self loops
    wl = W.make_workload(3, n=700)
    rp, col = orc.adjacency(wl.src, wl.dst, wl.n, wl.adj_flags)
    a = _dense_adj(wl.n, rp, col)
    assert np.all(np.diag(a) == 0) and np.array_equal(a, a.T)
    logits, hidden = orc.forward("sage", rp, col, wl.x, wl.layers, return_hidden=True)
    v = wl.x.astype(np.int64)
    for l, p in enumerate(wl.layers):
        k_in = v.shape[1]
        nb = np.where(a @ v >= p.t_agg[None, :], 1, -1)
        z = v @ p.w[:k_in].astype(np.int64) + nb @ p.w[k_in:].astype(np.int64)
        if p.alpha is None:
            v = np.where(z >= p.t_mm[None, :], 1, -1)
            assert np.array_equal(hidden[l], v)
        else:
            assert np.allclose(logits, p.alpha.astype(np.float64)[None, :] * z, rtol=1e-6, atol=0)
    iso = np.nonzero(orc.degrees(rp) == 0)[0]     # isolated node: S = 0, bit = (0 >= T)
    if len(iso):
        nb0 = orc.rebin(orc.spmm_pm1(rp, col, wl.x), wl.layers[0].t_agg)
        assert np.array_equal(nb0[iso[0]], np.where(0 >= wl.layers[0].t_agg, 1, -1))


# ---------------------------------------------------------------- Algorithm 1
def test_alg1_tile_set_count_example():
    # Section 3.3.2, steps 1-2: ten tiles make two tile groups of 8 slots
    assert alg1.TS == 8 and alg1.n_tile_sets(10) == 2 and alg1.n_tile_sets(8) == 1


@pytest.mark.parametrize("n,e,c,seed", [(7, 20, 32, 0), (30, 140, 40, 1), (45, 700, 64, 2)])
def test_alg1_emulator_equals_oracle(n, e, c, seed):
    r = _rng(seed)
    src, dst = W.random_graph(r, n, e)
    rp, col = orc.adjacency(src, dst, n, orc.ADJ_SYMMETRIZE | orc.ADJ_ADD_SELF_LOOPS)
    v = W.pm1(r, (n, c))
    n_words = (c + 31) // 32
    words = [[0] * n_words for _ in range(n)]
    for j in range(n):
        for ch in range(c):
            if v[j, ch] > 0:
                words[j][ch // 32] |= 1 << (ch % 32)
    frdc = alg1.build_frdc(n, rp, col)
    if n == 45:
        assert max(np.diff(frdc[0])) > alg1.TS        # more than one tile set
    out = alg1.bspmm_bbb(n, frdc, words, n_words)
    expect = orc.rebin(orc.spmm_pm1(rp, col, v), np.zeros(c, dtype=np.int32))
    for i in range(n):
        for ch in range(c):
            bit = (out[i][ch // 32] >> (ch % 32)) & 1
            assert bit == (1 if expect[i, ch] > 0 else 0)


# ------------------------------------------- weighted / full-precision aggregation
def _small_graph(seed, n=60, e=400, flags=W.ADJ_SYMMETRIZE | W.ADJ_ADD_SELF_LOOPS):
    r = _rng(seed)
    src, dst = W.random_graph(r, n, e)
    rp, col = orc.adjacency(src, dst, n, flags)
    return r, n, rp, col


def test_weighted_spmm_equals_dense_matmul_with_factor_vectors():
    """diag(r) A diag(f) X by numpy's dense float64 matmul (an independent routine);
    a transposed adjacency, a swapped r / f or a dropped factor fails it."""
    r, n, rp, col = _small_graph(1, flags=0)          # directed: A != A^T
    a = np.zeros((n, n))
    for i in range(n):
        a[i, col[rp[i]:rp[i + 1]]] = 1.0
    x = r.standard_normal((n, 9))
    rv, fv = r.uniform(0.5, 2.0, n), r.uniform(0.5, 2.0, n)
    want = (rv[:, None] * a * fv[None, :]) @ x
    assert np.allclose(orc.spmm_weighted(rp, col, x, rv, fv), want, rtol=1e-13, atol=1e-13)
    assert np.allclose(orc.spmm_weighted(rp, col, x, None, fv), (a * fv[None, :]) @ x,
                       rtol=1e-13, atol=1e-13)
    assert np.allclose(orc.spmm_weighted(rp, col, x, rv, None), (rv[:, None] * a) @ x,
                       rtol=1e-13, atol=1e-13)
    assert not np.allclose(orc.spmm_weighted(rp, col, x, fv, rv), want)


def test_weighted_spmm_unit_factors_on_pm1_is_the_integer_aggregation():
    """r = f = 1 on +-1 activations: both the float64 and the step-rounded float32 sum are
    the exact integers of the 0/1 x +-1 aggregation (Section 3.2.2)."""
    r, n, rp, col = _small_graph(2)
    v = W.pm1(r, (n, 33))
    s = orc.spmm_pm1(rp, col, v)
    assert np.array_equal(orc.spmm_weighted(rp, col, v), s.astype(np.float64))
    assert np.array_equal(orc.spmm_weighted_f32(rp, col, v), s.astype(np.float32))


def test_weighted_spmm_closed_forms_regular_graph_and_mean():
    """k-regular ring with self-loops, symmetric normalisation r = f = deg^-1/2: constant
    input 1 gives exactly 1 per node; mean (r = 1/deg) of a constant is the constant; the
    normalised operator is symmetric: <u, P v> = <P u, v>."""
    n, k = 40, 3
    src = np.repeat(np.arange(n), k).astype(np.int32)
    dst = ((src + np.tile(np.arange(1, k + 1), n)) % n).astype(np.int32)
    rp, col = orc.adjacency(src, dst, n, W.ADJ_SYMMETRIZE | W.ADJ_ADD_SELF_LOOPS)
    deg = orc.degrees(rp).astype(np.float64)
    assert np.all(deg == 2 * k + 1)
    dinv = deg ** -0.5
    ones = np.ones((n, 2))
    assert np.allclose(orc.spmm_weighted(rp, col, ones, dinv, dinv), 1.0, rtol=0, atol=1e-15)
    r, _, rp2, col2 = _small_graph(3)
    deg2 = orc.degrees(rp2).astype(np.float64)
    c = np.full((len(deg2), 3), 2.5)
    assert np.allclose(orc.spmm_weighted(rp2, col2, c, 1.0 / deg2, None), 2.5, rtol=1e-15)
    d2 = deg2 ** -0.5
    u, v = r.standard_normal((len(deg2), 1)), r.standard_normal((len(deg2), 1))
    pu, pv = orc.spmm_weighted(rp2, col2, u, d2, d2), orc.spmm_weighted(rp2, col2, v, d2, d2)
    assert abs(float((u * pv).sum() - (pu * v).sum())) < 1e-12


def test_weighted_spmm_f32_steps_handworked_and_error_bound():
    """Order and rounding of the float32 variant on a hand-worked row: (2^24 + 1) - 2^24
    summed left to right in float32 is 1 only if the big terms cancel first; and on random
    inputs the float32 value stays within deg * eps * sum|terms| of the float64 one."""
    rp = np.array([0, 3], dtype=np.int64)
    x = np.array([[16777216.0], [1.0], [-16777216.0]], dtype=np.float32)
    col = np.array([0, 1, 2], dtype=np.int32)       # 2^24 + 1 rounds to 2^24, then - 2^24 = 0
    assert orc.spmm_weighted_f32(rp, col, x)[0, 0] == 0.0
    col = np.array([0, 2, 1], dtype=np.int32)       # 2^24 - 2^24 + 1 = 1
    assert orc.spmm_weighted_f32(rp, col, x)[0, 0] == 1.0
    assert orc.spmm_weighted(rp, col, x)[0, 0] == 1.0
    f = np.array([3.0, 0.5, 3.0], dtype=np.float32)  # factors multiply the column, r the row
    assert orc.spmm_weighted_f32(rp, col, x, np.array([2.0], np.float32), f)[0, 0] == 1.0
    r, n, rp, col = _small_graph(4, n=200, e=4000)
    xx = r.standard_normal((n, 7)).astype(np.float32)
    fv = r.uniform(0.1, 1.0, n).astype(np.float32)
    rv = r.uniform(0.1, 1.0, n).astype(np.float32)
    y64 = orc.spmm_weighted(rp, col, xx, rv, fv)
    y32 = orc.spmm_weighted_f32(rp, col, xx, rv, fv)
    mag = orc.spmm_weighted(rp, col, np.abs(xx), rv, fv)
    deg = orc.degrees(rp)[:, None]
    assert np.all(np.abs(y32 - y64) <= (deg + 2) * 2.0 ** -24 * mag + 1e-30)
    tau = np.zeros(7, dtype=np.float32)
    assert np.array_equal(orc.rebin_f32(y32, tau), np.where(y32 >= 0, 1, -1))


def test_weighted_layers_reduce_to_the_integer_layers():
    """Unit factors and integer thresholds: the weighted GCN layer is the integer GCN layer.
    On a k-regular graph the mean aggregator with threshold tau is the sum aggregator with
    the integer threshold ceil(tau * k) (tau * k exact in float32)."""
    r, n, rp, col = _small_graph(11, n=80, e=600)
    v, w = W.pm1(r, (n, 20)), W.pm1(r, (20, 12))
    t_mm = r.integers(-3, 4, 12).astype(np.int32)
    t_agg = r.integers(-3, 4, 12).astype(np.int32)
    one = np.ones(n, dtype=np.float32)
    assert np.array_equal(
        orc.gcn_hidden_layer_norm(rp, col, v, w, t_mm, one, one, t_agg.astype(np.float32)),
        orc.gcn_hidden_layer(rp, col, v, w, t_mm, t_agg))
    n, k = 64, 4
    src = np.repeat(np.arange(n), k).astype(np.int32)
    dst = ((src + np.tile(np.arange(1, k + 1), n)) % n).astype(np.int32)
    rp, col = orc.adjacency(src, dst, n, W.ADJ_SYMMETRIZE)
    assert np.all(orc.degrees(rp) == 2 * k)
    v, w = W.pm1(r, (n, 10)), W.pm1(r, (20, 6))
    tau = np.array([-0.5, -0.25, 0.0, 0.125, 0.25, 0.5, -0.75, 0.75, 0.375, -0.125], np.float32)
    t_int = np.ceil(tau.astype(np.float64) * 2 * k).astype(np.int32)
    t_mm = r.integers(-2, 3, 6).astype(np.int32)
    rmean = np.full(n, 1.0 / (2 * k), dtype=np.float32)
    assert np.array_equal(orc.sage_hidden_layer_mean(rp, col, v, w, rmean, tau, t_mm),
                          orc.sage_hidden_layer(rp, col, v, w, t_int, t_mm))


def test_weighted_out_layer_reduces_to_the_integer_out_layer():
    """Unit factors, alpha = 1: the weighted output layer gives the integers of the exact
    output layer (small enough to be exact in float32)."""
    r, n, rp, col = _small_graph(12, n=70, e=500)
    v, w = W.pm1(r, (n, 24)), W.pm1(r, (24, 5))
    one = np.ones(5, dtype=np.float32)
    got = orc.gcn_out_layer_norm(rp, col, v, w, one, None, None)
    assert np.array_equal(got, orc.gcn_out_layer(rp, col, v, w, one))
    y64 = orc.spmm_weighted(rp, col, orc.bmm(v, w).astype(np.float64))
    assert np.array_equal(got.astype(np.float64), y64)


# ---------------------------------------------------------------------------
# ADD: the auxiliary merge (Section 3.1.2)
# ---------------------------------------------------------------------------

def test_add_handworked_values_and_float32_rounding():
    """ADD.BBF on +-1 tensors can only give -2, 0, 2; ADD.FFF is ONE float32 addition:
    hand-worked cases where float32 and wider arithmetic differ, written as literals."""
    a = np.array([[1, 1, -1, -1]], dtype=np.int8)
    b = np.array([[1, -1, 1, -1]], dtype=np.int8)
    assert orc.add_f32(a, b).tolist() == [[2.0, 0.0, 0.0, -2.0]]
    # 2^24 + 1 is not a float32: the sum rounds to even (2^24); 2^24 + 3 rounds up to 2^24 + 4
    fa = np.array([[16777216.0, 16777216.0, 0.1, -0.0]], dtype=np.float32)
    fb = np.array([[1.0, 3.0, 0.2, 0.0]], dtype=np.float32)
    got = orc.add_f32(fa, fb)
    assert got.dtype == np.float32
    assert got[0, 0] == 16777216.0 and got[0, 1] == 16777220.0
    # float32(0.1) + float32(0.2) rounded to float32: 0x3E99999A (0.3 in float64 arithmetic
    # would round to the same float32 here; the literal pins the bit pattern)
    assert got[0, 2].view(np.uint32) == 0x3E99999A
    assert got[0, 3] == 0.0
    # mixed operands: a binary tensor counts as +-1.0
    assert orc.add_f32(a, fb).tolist() == [[2.0, 4.0, np.float32(-1.0) + np.float32(0.2), -1.0]]


def test_add_is_commutative_and_exact_against_float64_when_representable():
    r = np.random.default_rng(5)
    a = r.integers(-1000, 1000, size=(50, 70)).astype(np.float32)
    b = r.integers(-1000, 1000, size=(50, 70)).astype(np.float32)
    s = orc.add_f32(a, b)
    assert np.array_equal(s, orc.add_f32(b, a))
    assert np.array_equal(s.astype(np.float64), a.astype(np.float64) + b.astype(np.float64))


def test_sage_layer_merged_by_addition_equals_the_concatenated_form():
    """X_i W1 + agg W2 (merge by ADD) and [X_i | agg] [W1; W2] (merge by CONCAT) are the
    same integers: pins the added form against the concatenated one, itself pinned above
    to the two-matmul form."""
    r = np.random.default_rng(11)
    n, k, m = 300, 70, 33
    src, dst = W.random_graph(r, n, 2000)
    rp, col = orc.adjacency(src, dst, n, W.ADJ_SYMMETRIZE)
    v = W.pm1(r, (n, k))
    w = W.pm1(r, (2 * k, m))
    t_agg = r.integers(-3, 4, size=k).astype(np.int32)
    t_mm = r.integers(-9, 10, size=m).astype(np.int32)
    cat = orc.sage_hidden_layer(rp, col, v, w, t_agg, t_mm)
    added = orc.sage_hidden_layer_added(rp, col, v, w[:k], w[k:], t_agg, t_mm)
    assert np.array_equal(cat, added)
    # and the float route the ADD.FFF function takes: scaled products added in float32
    nb = orc.rebin(orc.spmm_pm1(rp, col, v), t_agg)
    z1, z2 = orc.bmm(v, w[:k]), orc.bmm(nb, w[k:])
    y = orc.add_f32(z1.astype(np.float32), z2.astype(np.float32))      # small integers: exact
    assert np.array_equal(orc.rebin_f32(y, t_mm.astype(np.float32)), cat)


# ---------------------------------------------------------------------------
# full-precision aggregation recipe (Table 3, "Ours (full)")
# ---------------------------------------------------------------------------

def test_full_precision_aggregation_layer_special_cases():
    """(1) Unit scale, unit factors, integer thresholds: the float layer is the integer layer
    (all values are small integers, exact in float32).  (2) The redundant-scale remark of
    Section 3.1.1: a positive scale in front of BIN changes nothing -- with power-of-two
    scales (exact in float32) and thresholds scaled alike the bits are identical.  (3) The
    weighted case against the float64 definition away from the thresholds."""
    r = np.random.default_rng(21)
    n, k, m = 400, 90, 37
    src, dst = W.random_graph(r, n, 3000)
    rp, col = orc.adjacency(src, dst, n, W.ADJ_SYMMETRIZE | W.ADJ_ADD_SELF_LOOPS)
    v = W.pm1(r, (n, k))
    w = W.pm1(r, (k, m))
    t = r.integers(-40, 41, size=m).astype(np.int32)
    ones = np.ones(m, dtype=np.float32)
    # (1): no binarization between product and aggregation: out = (A (v W) >= t)
    want = orc.rebin(orc.spmm_i64(rp, col, orc.bmm(v, w)), t)
    got = orc.gcn_hidden_layer_full(rp, col, v, w, ones, None, None, t.astype(np.float32))
    assert np.array_equal(got, want)
    # (2): per-channel positive power-of-two scales
    alpha = (2.0 ** r.integers(-3, 4, size=m)).astype(np.float32)
    got2 = orc.gcn_hidden_layer_full(rp, col, v, w, alpha, None, None,
                                     alpha * t.astype(np.float32))
    assert np.array_equal(got2, want)
    # (3): symmetric normalisation, float64 definition; entries within the float32 error
    # bound of their threshold are not compared
    deg = orc.degrees(rp).astype(np.float64)
    dinv = deg ** -0.5
    z64 = orc.bmm(v, w).astype(np.float64) * alpha.astype(np.float64)
    y64 = orc.spmm_weighted(rp, col, z64, dinv, dinv)
    tau = r.standard_normal(m).astype(np.float32)
    got3 = orc.gcn_hidden_layer_full(rp, col, v, w, alpha, dinv.astype(np.float32),
                                     dinv.astype(np.float32), tau)
    mag = orc.spmm_weighted(rp, col, np.abs(z64), dinv, dinv)
    safe = np.abs(y64 - tau) > (deg[:, None] + 6) * 2.0 ** -23 * mag + 1e-30
    assert safe.mean() > 0.9
    assert np.array_equal(got3[safe], np.where(y64 >= tau, 1, -1).astype(np.int8)[safe])
