"""GPU parity: every kernel of the library against the CPU oracle, element by
element, on the same seeded inputs.  Integers, packed words and indices must be
bit-exact; float logits within 1e-5 relative (one float multiply per logit)."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2305_02522_amd import workloads as W

pytestmark = pytest.mark.gpu

SYM_LOOPS = W.ADJ_SYMMETRIZE | W.ADJ_ADD_SELF_LOOPS


@pytest.fixture(scope="module")
def B():
    from paper_2305_02522_amd import binding
    return binding


@pytest.fixture(scope="module")
def ctx(B):
    c = B.Context(0)
    yield c
    c.close()


TUNINGS = {"default": (10208, 255, 8), "csr-only": (10208, 255, 1 << 30),
           "blocked-small": (128, 16, 0), "blocked-long-parts": (64, 1023, 0),
           "blocked-odd": (1000, 100, 0), "blocked-default-sizes": (8192, 512, 0),
           "blocked-largest-block": (10208, 255, 0)}


@pytest.fixture(scope="module", params=["auto", "valu", "mfma"])
def gemm_ctx(request, B):
    """Contexts that choose the BMM kernel per shape, or always take the VALU / the
    matrix-core kernel (the latter falls back when the weights do not fit in LDS)."""
    c = B.Context(0)
    B.ctx_set_bgemm_path(c, {"auto": B.BGEMM_AUTO, "valu": B.BGEMM_VALU,
                             "mfma": B.BGEMM_MFMA}[request.param])
    yield c
    c.close()


@pytest.fixture(params=list(TUNINGS))
def tuned(request, B, ctx):
    """Every aggregation test runs on the CSR path and on the column-blocked path
    with several block / part sizes: results must not depend on the format."""
    B.ctx_set_tuning(ctx, *TUNINGS[request.param])
    yield request.param
    B.ctx_set_tuning(ctx, *TUNINGS["default"])


def dev(a):
    return torch.as_tensor(np.ascontiguousarray(a), device="cuda")


def words_np(t):
    """int64 torch tensor of packed words -> uint64 numpy."""
    return t.cpu().numpy().view(np.uint64)


def rel_close(got, ref, tol=1e-5):
    denom = np.maximum(np.abs(ref), 1e-30)
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64)) / denom
    err[got == ref] = 0
    return err.max() <= tol


# ------------------------------------------------------------------ a1: pack
@pytest.mark.parametrize("n,K,pad_ld,pad_out", [
    (1, 1, 0, 0), (3, 63, 0, 0), (5, 64, 3, 1), (130, 65, 0, 0), (257, 100, 4, 2),
    (1000, 602, 0, 0), (2708, 1433, 0, 0), (64, 4096, 0, 0), (70001, 128, 0, 0),
    # rows of fewer than 4 elements (one element per lane), rows that end inside a lane's 4
    # elements (the load is moved back and the nibble shifted), rows at odd element offsets
    (7, 2, 1, 0), (9, 3, 0, 1), (33, 4, 1, 0), (33, 5, 0, 0), (100, 6, 3, 0), (100, 7, 0, 0),
    (257, 66, 1, 0), (300, 67, 0, 2), (129, 127, 1, 0), (50, 129, 2, 0), (1025, 191, 5, 0)])
def test_pack_f32(B, ctx, n, K, pad_ld, pad_out):
    r = np.random.default_rng(n * 7919 + K)
    ldx = K + pad_ld
    x = r.standard_normal((n, ldx)).astype(np.float32)
    x[r.random((n, ldx)) < 0.05] = 0.0           # exact ties
    x[r.random((n, ldx)) < 0.02] = -0.0
    kw = (K + 63) // 64
    stride = kw + pad_out
    out = torch.full((n, stride), -1, dtype=torch.int64, device="cuda")
    B.pack_f32(ctx, dev(x), n, K, ldx, None, out, stride)
    torch.cuda.synchronize()
    ref = orc.to_words(orc.bin_f32(x[:, :K]))
    got = words_np(out)
    assert np.array_equal(got[:, :kw], ref)
    assert np.all(got[:, kw:] == np.uint64(0xFFFFFFFFFFFFFFFF))      # untouched
    # per-column threshold (folded BatchNorm)
    tau = r.standard_normal(K).astype(np.float32)
    x[:, :K][r.random((n, K)) < 0.05] = 0
    x[0, :K] = tau                                                     # ties -> +1
    B.pack_f32(ctx, dev(x), n, K, ldx, dev(tau), out, stride)
    torch.cuda.synchronize()
    assert np.array_equal(words_np(out)[:, :kw], orc.to_words(orc.bin_f32(x[:, :K], tau)))


@pytest.mark.parametrize("n,K", [(1, 1), (77, 100), (300, 1433), (5000, 64), (40, 3), (41, 5),
                                 (300, 66), (123, 130)])
def test_pack_i8_and_weights(B, ctx, n, K):
    r = np.random.default_rng(K)
    x = r.integers(-128, 128, size=(n, K), dtype=np.int8)
    kw = (K + 63) // 64
    out = torch.zeros((n, kw), dtype=torch.int64, device="cuda")
    B.pack_i8(ctx, dev(x), n, K, K, out, kw)
    torch.cuda.synchronize()
    assert np.array_equal(words_np(out), orc.to_words(orc.bin_i8(x)))
    # weights: transposed packing, w is [K][M]
    M = 37
    w = W.pm1(r, (K, M))
    wb = torch.zeros((M, kw + 1), dtype=torch.int64, device="cuda")
    B.pack_weights_i8(ctx, dev(w), K, M, M, wb, kw + 1)
    torch.cuda.synchronize()
    assert np.array_equal(words_np(wb)[:, :kw], orc.to_words(np.ascontiguousarray(w.T)))


# ------------------------------------------------------------------ a2: adjacency
def _csr_from_gpu(B, adj):
    import ctypes
    rp_p, col_p, deg_p = adj.csr_pointers()
    n, nnz = adj.n, adj.nnz
    rp = torch.empty(n + 1, dtype=torch.int32, device="cuda")
    col = torch.empty(max(nnz, 1), dtype=torch.int32, device="cuda")
    deg = torch.empty(n, dtype=torch.int32, device="cuda")
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
    assert hip.hipMemcpy(rp.data_ptr(), rp_p, 4 * (n + 1), 3) == 0
    if nnz:
        assert hip.hipMemcpy(col.data_ptr(), col_p, 4 * nnz, 3) == 0
    assert hip.hipMemcpy(deg.data_ptr(), deg_p, 4 * n, 3) == 0
    torch.cuda.synchronize()
    return (rp.cpu().numpy().view(np.uint32).astype(np.int64), col.cpu().numpy()[:nnz],
            deg.cpu().numpy())


@pytest.mark.parametrize("n,e,flags,seed", [
    (1, 0, 0, 0), (1, 0, W.ADJ_ADD_SELF_LOOPS, 0), (5, 0, 0, 1), (7, 30, 0, 2),
    (100, 1000, W.ADJ_SYMMETRIZE, 3), (1000, 5000, SYM_LOOPS, 4),
    (4097, 70000, SYM_LOOPS, 5), (300000, 900000, SYM_LOOPS, 6), (50, 20000, SYM_LOOPS, 7)])
def test_adj_build_matches_set_definition(B, ctx, n, e, flags, seed):
    r = np.random.default_rng(seed)
    src, dst = W.random_graph(r, n, e)
    s = dev(src) if e else None
    d = dev(dst) if e else None
    adj = B.adj_build(ctx, s, d, e, n, flags)
    rp_ref, col_ref = orc.adjacency(src, dst, n, flags)
    rp, col, deg = _csr_from_gpu(B, adj)
    assert adj.nnz == rp_ref[-1]
    assert np.array_equal(rp, rp_ref)
    assert np.array_equal(col, col_ref)
    assert np.array_equal(deg, orc.degrees(rp_ref))
    assert adj.max_degree == (orc.degrees(rp_ref).max() if n else 0)
    adj.close()


def test_tuning_validation(B, ctx):
    for bad in ((63, 512, 32), (10209, 512, 32), (8192, 3, 32), (8192, 1024, 32), (8192, 512, -1)):
        with pytest.raises(B.BitgnnError) as e:
            B.ctx_set_tuning(ctx, *bad)
        assert e.value.code == B.ERR_INVALID_ARG
    B.ctx_set_tuning(ctx, *TUNINGS["default"])


def test_adj_build_rejects_out_of_range(B, ctx):
    src = dev(np.array([0, 1, 5], dtype=np.int32))
    dst = dev(np.array([1, 2, 0], dtype=np.int32))
    with pytest.raises(B.BitgnnError) as e:
        B.adj_build(ctx, src, dst, 3, 5, 0)
    assert e.value.code == B.ERR_INDEX_RANGE
    src = dev(np.array([0, -1], dtype=np.int32))
    dst = dev(np.array([1, 2], dtype=np.int32))
    with pytest.raises(B.BitgnnError) as e:
        B.adj_build(ctx, src, dst, 2, 5, 0)
    assert e.value.code == B.ERR_INDEX_RANGE


# ------------------------------------------------------------------ a3: BGEMM
def _pack_host(v):
    return dev(orc.to_words(v).view(np.int64))


@pytest.mark.parametrize("n,K,M", [
    (1, 1, 1), (5, 63, 7), (129, 64, 64), (300, 65, 65), (1000, 100, 41), (777, 602, 128),
    (500, 1433, 64), (2048, 512, 256), (100, 1000, 47), (4099, 128, 40), (33, 2100, 130),
    (5000, 200, 256), (6000, 512, 47), (4500, 64, 33), (300, 96, 528),
    # matrix-core kernel in column chunks: 2 x 128, 128 + 128 + 44, 256 + 256 + 88
    (1500, 1000, 256), (700, 1000, 300), (400, 512, 600)])
def test_bgemm_three_epilogues(B, gemm_ctx, n, K, M):
    ctx = gemm_ctx
    r = np.random.default_rng(K * 1000 + M)
    x = W.pm1(r, (n, K))
    w = W.pm1(r, (K, M))
    z = orc.bmm(x, w)
    kw = (K + 63) // 64
    xb = _pack_host(x)
    wb = _pack_host(np.ascontiguousarray(w.T))
    # RAW
    out = torch.full((n, M + 3), 12345, dtype=torch.int32, device="cuda")
    B.bgemm(ctx, xb, n, kw, K, kw, wb, M, kw, B.EPI_RAW_I32, None, None, out, M + 3)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(got[:, :M], z)
    assert np.all(got[:, M:] == 12345)
    # THRESH
    t = r.integers(-6, 7, size=M).astype(np.int32)
    mw = (M + 63) // 64
    ob = torch.full((n, mw), -1, dtype=torch.int64, device="cuda")
    B.bgemm(ctx, xb, n, kw, K, kw, wb, M, kw, B.EPI_THRESH_BITS, dev(t), None, ob, mw)
    torch.cuda.synchronize()
    assert np.array_equal(words_np(ob), orc.to_words(orc.rebin(z, t)))       # pad bits 0
    # thresholds at and beyond the range of Z (|Z| <= K) and at the int32 limits
    ext = np.array([np.iinfo(np.int32).min, np.iinfo(np.int32).max, K + 1, -K - 1, K, -K,
                    np.iinfo(np.int32).max - 1, np.iinfo(np.int32).min + 1], dtype=np.int64)
    t2 = ext[r.integers(0, len(ext), size=M)].astype(np.int32)
    ob.fill_(-1)
    B.bgemm(ctx, xb, n, kw, K, kw, wb, M, kw, B.EPI_THRESH_BITS, dev(t2), None, ob, mw)
    torch.cuda.synchronize()
    assert np.array_equal(words_np(ob), orc.to_words(orc.rebin(z, t2)))
    # SCALE
    alpha = r.uniform(0.5, 1.5, M).astype(np.float32)
    of = torch.zeros((n, M), dtype=torch.float32, device="cuda")
    B.bgemm(ctx, xb, n, kw, K, kw, wb, M, kw, B.EPI_SCALE_F32, None, dev(alpha), of, M)
    torch.cuda.synchronize()
    assert rel_close(of.cpu().numpy(), orc.scale(z, alpha))


@pytest.mark.parametrize("n,K,M", [(1, 1, 1), (70, 63, 7), (300, 65, 65), (1000, 602, 128),
                                   (500, 1433, 64), (129, 512, 256), (257, 100, 300),
                                   (4099, 130, 41)])
def test_bgemm_f32_binarizes_inside(B, ctx, n, K, M):
    r = np.random.default_rng(K * 31 + M)
    ldx = K + (3 if K % 2 else 0)
    x = r.standard_normal((n, ldx)).astype(np.float32)
    x[r.random((n, ldx)) < 0.05] = 0.0
    x[r.random((n, ldx)) < 0.02] = -0.0
    w = W.pm1(r, (K, M))
    kw = (K + 63) // 64
    wb = _pack_host(np.ascontiguousarray(w.T))
    for tau in (None, r.standard_normal(K).astype(np.float32)):
        if tau is not None:
            x[0, :K] = tau
        v = orc.bin_f32(x[:, :K], tau)
        z = orc.bmm(v, w)
        out = torch.full((n, M + 1), 5, dtype=torch.int32, device="cuda")
        B.bgemm_f32(ctx, dev(x), n, K, ldx, None if tau is None else dev(tau), wb, M, kw,
                    B.EPI_RAW_I32, None, None, out, M + 1)
        t = r.integers(-6, 7, size=M).astype(np.int32)
        mw = (M + 63) // 64
        ob = torch.full((n, mw), -1, dtype=torch.int64, device="cuda")
        B.bgemm_f32(ctx, dev(x), n, K, ldx, None if tau is None else dev(tau), wb, M, kw,
                    B.EPI_THRESH_BITS, dev(t), None, ob, mw)
        alpha = r.uniform(0.5, 1.5, M).astype(np.float32)
        of = torch.zeros((n, M), dtype=torch.float32, device="cuda")
        B.bgemm_f32(ctx, dev(x), n, K, ldx, None if tau is None else dev(tau), wb, M, kw,
                    B.EPI_SCALE_F32, None, dev(alpha), of, M)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert np.array_equal(got[:, :M], z) and np.all(got[:, M] == 5)
        assert np.array_equal(words_np(ob), orc.to_words(orc.rebin(z, t)))
        assert rel_close(of.cpu().numpy(), orc.scale(z, alpha))


def test_bgemm_segmented_k_with_interior_pad_bits(B, gemm_ctx):
    ctx = gemm_ctx
    # [self | nbr] rows: two 100-bit segments, each padded to 128 bits, K = 200
    r = np.random.default_rng(99)
    n, k_in, M = 300, 100, 70
    a, b = W.pm1(r, (n, k_in)), W.pm1(r, (n, k_in))
    w = W.pm1(r, (2 * k_in, M))
    z = orc.bmm(orc.concat(a, b), w)
    xb = dev(np.concatenate([orc.to_words(a), orc.to_words(b)], axis=1).view(np.int64))
    wt = np.ascontiguousarray(w.T)
    wb = dev(np.concatenate([orc.to_words(wt[:, :k_in]), orc.to_words(wt[:, k_in:])],
                            axis=1).view(np.int64))
    out = torch.zeros((n, M), dtype=torch.int32, device="cuda")
    B.bgemm(ctx, xb, n, 4, 2 * k_in, 4, wb, M, 4, B.EPI_RAW_I32, None, None, out, M)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), z)


# ------------------------------------------------------------------ a4: bit-SpMM
def _graph(B, ctx, n, e, flags, seed, hubs=0):
    r = np.random.default_rng(seed)
    src, dst = W.random_graph(r, n, e)
    if hubs:                     # a few very long rows
        hs = r.integers(0, n, size=hubs * n // 2, dtype=np.int32) % max(hubs, 1)
        hd = r.integers(0, n, size=hubs * n // 2, dtype=np.int32)
        src, dst = np.concatenate([src, hs]), np.concatenate([dst, hd])
    adj = B.adj_build(ctx, dev(src), dev(dst), len(src), n, flags)
    rp, col = orc.adjacency(src, dst, n, flags)
    return adj, rp, col, r


@pytest.mark.parametrize("n,e,C,flags,hubs", [
    (1, 0, 1, W.ADJ_ADD_SELF_LOOPS, 0), (9, 20, 7, SYM_LOOPS, 0), (100, 700, 32, SYM_LOOPS, 0),
    (257, 3000, 33, W.ADJ_SYMMETRIZE, 0), (1000, 20000, 64, SYM_LOOPS, 0),
    (3000, 40000, 100, W.ADJ_SYMMETRIZE, 0), (5000, 100000, 128, SYM_LOOPS, 2),
    (2000, 30000, 256, SYM_LOOPS, 0), (1500, 9000, 500, W.ADJ_SYMMETRIZE, 0),
    (40000, 100000, 128, SYM_LOOPS, 1), (700, 300, 65, 0, 0),
    (70000, 200000, 96, SYM_LOOPS, 0),       # CSR path with the degree-ordered gather table
    (200000, 1000000, 64, SYM_LOOPS, 0)])    # blocked path with work items of 8 slices
def test_bspmm_raw_and_threshold(B, ctx, tuned, n, e, C, flags, hubs):
    adj, rp, col, r = _graph(B, ctx, n, e, flags, n + C, hubs)
    v = W.pm1(r, (n, C))
    s = orc.spmm_pm1(rp, col, v)
    cw = (C + 63) // 64
    hb = _pack_host(v)
    raw = torch.full((n, C + 1), 777, dtype=torch.int32, device="cuda")
    B.bspmm(ctx, adj, hb, C, cw, B.EPI_RAW_I32, None, raw, C + 1)
    torch.cuda.synchronize()
    got = raw.cpu().numpy()
    assert np.array_equal(got[:, :C], s)
    assert np.all(got[:, C] == 777)
    for t in (np.zeros(C, dtype=np.int32),                       # the paper's c >= 0
              r.integers(-4, 5, size=C).astype(np.int32),
              r.integers(-40000, 40000, size=C).astype(np.int32),
              np.full(C, 2**31 - 1, dtype=np.int32), np.full(C, -2**31, dtype=np.int32)):
        ob = torch.full((n, cw + 1), -1, dtype=torch.int64, device="cuda")
        B.bspmm(ctx, adj, hb, C, cw, B.EPI_THRESH_BITS, dev(t), ob, cw + 1)
        torch.cuda.synchronize()
        gw = words_np(ob)
        assert np.array_equal(gw[:, :cw], orc.to_words(orc.rebin(s, t)))
        assert np.all(gw[:, cw] == np.uint64(0xFFFFFFFFFFFFFFFF))
    adj.close()


def test_bspmm_star_graph_long_row(B, ctx, tuned):
    # one row with 70,000 neighbours: needs the 20-plane counters
    n, C = 70001, 96
    src = np.zeros(n - 1, dtype=np.int32)
    dst = np.arange(1, n, dtype=np.int32)
    adj = B.adj_build(ctx, dev(src), dev(dst), n - 1, n, SYM_LOOPS)
    rp, col = orc.adjacency(src, dst, n, SYM_LOOPS)
    assert adj.max_degree == n
    r = np.random.default_rng(5)
    v = (r.random((n, C)) < 0.5003).astype(np.int8) * 2 - 1
    s = orc.spmm_pm1(rp, col, v)
    t = r.integers(-300, 300, size=C).astype(np.int32)
    ob = torch.zeros((n, 2), dtype=torch.int64, device="cuda")
    B.bspmm(ctx, adj, _pack_host(v), C, 2, B.EPI_THRESH_BITS, dev(t), ob, 2)
    raw = torch.zeros((n, C), dtype=torch.int32, device="cuda")
    B.bspmm(ctx, adj, _pack_host(v), C, 2, B.EPI_RAW_I32, None, raw, C)
    torch.cuda.synchronize()
    assert np.array_equal(raw.cpu().numpy(), s)
    assert np.array_equal(words_np(ob), orc.to_words(orc.rebin(s, t)))
    adj.close()


def test_adj_tune_measures_both_kernels_and_keeps_results(B, ctx):
    """The tuning utility times both aggregation kernels and records a preference; the
    aggregation gives the same bits before and after, whichever kernel won."""
    adj, rp, col, r = _graph(B, ctx, 20000, 400000, SYM_LOOPS, 77)
    assert adj.blocked_info()["parts"] > 0
    C = 128
    v = W.pm1(r, (20000, C))
    t = r.integers(-4, 5, size=C).astype(np.int32)
    want = orc.to_words(orc.rebin(orc.spmm_pm1(rp, col, v), t))
    hb = _pack_host(v)
    for step in range(2):
        ob = torch.zeros((20000, 2), dtype=torch.int64, device="cuda")
        B.bspmm(ctx, adj, hb, C, 2, B.EPI_THRESH_BITS, dev(t), ob, 2)
        torch.cuda.synchronize()
        assert np.array_equal(words_np(ob), want)
        if step == 0:
            csr_ms, blk_ms = B.adj_tune(ctx, adj, C, 3)
            assert csr_ms > 0 and blk_ms > 0
    with pytest.raises(B.BitgnnError) as ex:
        B.adj_tune(ctx, adj, 0, 3)
    assert ex.value.code == B.ERR_INVALID_ARG
    adj.close()
    sparse, _, _, _ = _graph(B, ctx, 3000, 6000, SYM_LOOPS, 78)     # CSR only: nothing to choose
    csr_ms, blk_ms = B.adj_tune(ctx, sparse, 64, 2)
    assert csr_ms > 0 and blk_ms == -1.0
    sparse.close()


# ------------------------------------------------------------------ a5: integer aggregation
def test_gcn_layer_tune_measures_both_recipes(B, ctx):
    adj, rp, col, r = _graph(B, ctx, 5000, 60000, SYM_LOOPS, 12)
    bin_ms, full_ms = B.gcn_layer_tune(ctx, adj, 100, 70, reps=2)
    assert 0.0 < bin_ms < 100.0 and 0.0 < full_ms < 100.0
    with pytest.raises(B.BitgnnError):
        B.gcn_layer_tune(ctx, adj, 100, 70, reps=0)
    adj.close()


@pytest.mark.parametrize("n,e,M,hubs", [
    (50, 200, 1, 0), (1000, 9000, 7, 0), (3000, 50000, 41, 0), (500, 4000, 64, 0),
    (300, 2000, 130, 0),
    (3000, 30000, 40, 1),      # 16-byte reads, 6 neighbours per gather, rows longer than a segment
    (2000, 20000, 128, 1),     # 16-byte reads, 2 neighbours per gather
    (2500, 30000, 34, 0),      # 8-byte reads
    (4000, 20000, 7, 2)])      # narrow rows with split rows
def test_spmm_i32(B, ctx, n, e, M, hubs):
    adj, rp, col, r = _graph(B, ctx, n, e, SYM_LOOPS, n + M, hubs)
    z = r.integers(-600, 601, size=(n, M)).astype(np.int32)
    y = orc.spmm_i64(rp, col, z)
    out = torch.zeros((n, M), dtype=torch.int32, device="cuda")
    B.spmm_i32(ctx, adj, dev(z), M, M, 600, None, out, M)
    alpha = r.uniform(0.5, 1.5, M).astype(np.float32)
    of = torch.zeros((n, M), dtype=torch.float32, device="cuda")
    B.spmm_i32(ctx, adj, dev(z), M, M, 600, dev(alpha), of, M)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), y)
    assert rel_close(of.cpu().numpy(), orc.scale(y, alpha))
    with pytest.raises(B.BitgnnError) as ex:
        B.spmm_i32(ctx, adj, dev(z), M, M, 2**31 - 1, None, out, M)
    assert ex.value.code == B.ERR_RANGE
    adj.close()


# ------------------------------------------- weighted / full-precision aggregation
@pytest.mark.parametrize("n,e,C,flags,hubs", [
    (1, 0, 1, W.ADJ_ADD_SELF_LOOPS, 0), (9, 20, 7, SYM_LOOPS, 0), (257, 3000, 33, W.ADJ_SYMMETRIZE, 0),
    (1000, 20000, 64, SYM_LOOPS, 0), (3000, 40000, 100, 0, 0), (5000, 100000, 128, SYM_LOOPS, 2),
    (1500, 9000, 300, W.ADJ_SYMMETRIZE, 0), (700, 300, 65, 0, 0)])
def test_spmm_f32_variants(B, ctx, n, e, C, flags, hubs):
    """Float and bit activations, with and without factor vectors (symmetric normalisation,
    mean), float and re-binarized output.  The float output must equal the step-rounded
    float32 oracle bit for bit (same order, same roundings) and lie within the bound
    (deg + 2) * 2^-24 * sum|terms| of the float64 definition; the bits are compared after
    the same float32 decision."""
    adj, rp, col, r = _graph(B, ctx, n, e, flags, n + C + 1, hubs)
    deg = np.maximum(orc.degrees(rp), 1).astype(np.float64)
    dinv = (deg ** -0.5).astype(np.float32)
    mean = (1.0 / deg).astype(np.float32)
    xf = r.standard_normal((n, C)).astype(np.float32)
    v = W.pm1(r, (n, C))
    cw = (C + 63) // 64
    tau = r.uniform(-0.5, 0.5, C).astype(np.float32)
    for x_bits, rv, fv in ((False, None, None), (False, dinv, dinv), (False, mean, None),
                           (True, dinv, dinv), (True, None, None), (True, mean, None)):
        x_host = v.astype(np.float32) if x_bits else xf
        x_dev = _pack_host(v) if x_bits else dev(xf)
        ldx = cw if x_bits else C
        want32 = orc.spmm_weighted_f32(rp, col, x_host, rv, fv)
        want64 = orc.spmm_weighted(rp, col, x_host, rv, fv)
        mag = orc.spmm_weighted(rp, col, np.abs(x_host), rv, fv)
        out = torch.full((n, C + 3), 777.0, dtype=torch.float32, device="cuda")
        B.spmm_f32(ctx, adj, x_dev, x_bits, C, ldx, None if rv is None else dev(rv),
                   None if fv is None else dev(fv), B.EPI_SCALE_F32, None, out, C + 3)
        ob = torch.full((n, cw + 1), -1, dtype=torch.int64, device="cuda")
        B.spmm_f32(ctx, adj, x_dev, x_bits, C, ldx, None if rv is None else dev(rv),
                   None if fv is None else dev(fv), B.EPI_THRESH_BITS, dev(tau), ob, cw + 1)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert np.array_equal(got[:, :C], want32)
        assert np.all(got[:, C:] == 777.0)
        bound = (orc.degrees(rp)[:, None] + 2) * 2.0 ** -24 * mag + 1e-30
        assert np.all(np.abs(got[:, :C].astype(np.float64) - want64) <= bound)
        gb = words_np(ob)
        assert np.array_equal(gb[:, :cw], orc.to_words(orc.rebin_f32(want32, tau)))
        assert np.all(gb[:, cw] == np.uint64(0xFFFFFFFFFFFFFFFF))
        if x_bits and rv is None:      # unit factors on bits: the exact integers of the bit path
            assert np.array_equal(got[:, :C], orc.spmm_pm1(rp, col, v).astype(np.float32))
    adj.close()


@pytest.mark.parametrize("n,e,C,hubs", [(1, 0, 1, 0), (300, 2500, 41, 0), (3000, 40000, 128, 1),
                                        (5000, 30000, 300, 0)])
def test_spmm_i16_scaled_integers(B, ctx, n, e, C, hubs):
    """Aggregation of alpha .* z from int16 rows: bit for bit the aggregation of the float
    rows the BMM's scale epilogue would have stored (the oracle scales, then sums)."""
    adj, rp, col, r = _graph(B, ctx, n, e, SYM_LOOPS, 40 + n, hubs)
    z = r.integers(-1500, 1501, size=(n, C)).astype(np.int16)
    z[0, 0], z[-1, -1] = 32767, -32768
    alpha = r.uniform(0.5, 1.5, size=C).astype(np.float32)
    dinv = (orc.degrees(rp).astype(np.float64) ** -0.5).astype(np.float32)
    want = orc.spmm_weighted_f32(rp, col, orc.scale(z.astype(np.int64), alpha), dinv, dinv)
    ldz = C + 2 + (C & 1)                                     # padded, even
    zd = dev(np.pad(z, ((0, 0), (0, ldz - C))))
    out = torch.full((n, C + 1), 7.0, dtype=torch.float32, device="cuda")
    B.spmm_i16(ctx, adj, zd, C, ldz, dev(alpha), dev(dinv), dev(dinv), B.EPI_SCALE_F32, None, out,
               C + 1)
    tau = (r.standard_normal(C) * 3).astype(np.float32)
    cw = (C + 63) // 64
    ob = torch.zeros((n, cw), dtype=torch.int64, device="cuda")
    B.spmm_i16(ctx, adj, zd, C, ldz, dev(alpha), dev(dinv), dev(dinv), B.EPI_THRESH_BITS, dev(tau),
               ob, cw)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(got[:, :C].view(np.uint32), want.view(np.uint32))
    assert np.all(got[:, C] == 7.0)
    assert np.array_equal(words_np(ob), orc.to_words(orc.rebin_f32(want, tau)))
    with pytest.raises(B.BitgnnError) as e:
        B.spmm_i16(ctx, adj, zd, C, ldz, None, None, None, B.EPI_SCALE_F32, None, out, C + 1)
    assert e.value.code == B.ERR_INVALID_ARG
    adj.close()


def test_spmm_f32_rejects_bad_arguments(B, ctx):
    adj, rp, col, r = _graph(B, ctx, 50, 200, SYM_LOOPS, 5)
    x = torch.zeros((50, 8), dtype=torch.float32, device="cuda")
    out = torch.zeros((50, 8), dtype=torch.float32, device="cuda")
    for args, code in (((x, 0, 8, 7, None, None, B.EPI_SCALE_F32, None, out, 8), B.ERR_INVALID_ARG),
                       ((x, 0, 8, 8, None, None, B.EPI_RAW_I32, None, out, 8), B.ERR_INVALID_ARG),
                       ((x, 0, 8, 8, None, None, B.EPI_THRESH_BITS, None, out, 8), B.ERR_INVALID_ARG),
                       ((x.data_ptr() + 2, 0, 8, 8, None, None, B.EPI_SCALE_F32, None, out, 8),
                        B.ERR_ALIGNMENT)):
        with pytest.raises(B.BitgnnError) as ex:
            B.spmm_f32(ctx, adj, *args)
        assert ex.value.code == code
    adj.close()


# ------------------------------------------------------------------ ADD (auxiliary merge)
@pytest.mark.parametrize("n,C", [(1, 1), (77, 64), (300, 65), (5000, 200), (20000, 128)])
@pytest.mark.parametrize("a_bits,b_bits", [(False, False), (True, True), (True, False),
                                           (False, True)])
def test_add_variants(B, ctx, n, C, a_bits, b_bits):
    """ADD.FFF, ADD.BBF and the mixed forms, float result bit for bit and binarized again."""
    r = np.random.default_rng(n * 7 + C)
    wds = (C + 63) // 64

    def operand(bits):
        if bits:
            v = W.pm1(r, (n, C))
            return v, dev(orc.to_words(v).view(np.int64)), wds
        f = r.standard_normal((n, C + 3)).astype(np.float32)[:, :C]      # padded leading dim
        f[r.random((n, C)) < 0.1] = 0.0
        d = dev(np.ascontiguousarray(np.pad(f, ((0, 0), (0, 3)))))
        return f, d, C + 3

    a, ad, lda = operand(a_bits)
    b, bd, ldb = operand(b_bits)
    want = orc.add_f32(a, b)
    out = torch.full((n, C + 1), 7.0, dtype=torch.float32, device="cuda")
    B.add(ctx, ad, a_bits, lda, bd, b_bits, ldb, n, C, B.EPI_SCALE_F32, None, out, C + 1)
    tau = r.standard_normal(C).astype(np.float32)
    tau[::3] = 0.0
    ob = torch.full((n, wds + 1), -1, dtype=torch.int64, device="cuda")
    B.add(ctx, ad, a_bits, lda, bd, b_bits, ldb, n, C, B.EPI_THRESH_BITS, dev(tau), ob, wds + 1)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(got[:, :C].view(np.uint32), want.view(np.uint32))
    assert np.all(got[:, C] == 7.0)                                       # padding untouched
    gb = words_np(ob)
    assert np.array_equal(gb[:, :wds], orc.to_words(orc.rebin_f32(want, tau)))
    assert np.all(gb[:, wds] == np.uint64(0xFFFFFFFFFFFFFFFF))


def test_add_merges_a_sage_layer_like_the_concatenated_form(B, ctx):
    """ADD.FFF on the two scaled products of a GraphSAGE layer, binarized: the bits of the
    library's concatenated layer."""
    n, e, k, m = 3000, 30000, 100, 70
    adj, rp, col, r = _graph(B, ctx, n, e, W.ADJ_SYMMETRIZE, 31)
    v = W.pm1(r, (n, k))
    w = W.pm1(r, (2 * k, m))
    t_agg = r.integers(-3, 4, size=k).astype(np.int32)
    t_mm = r.integers(-9, 10, size=m).astype(np.int32)
    want = orc.sage_hidden_layer_added(rp, col, v, w[:k], w[k:], t_agg, t_mm)
    kw, mw = (k + 63) // 64, (m + 63) // 64
    vb = dev(orc.to_words(v).view(np.int64))
    nb = torch.zeros((n, kw), dtype=torch.int64, device="cuda")
    B.bspmm(ctx, adj, vb, k, kw, B.EPI_THRESH_BITS, dev(t_agg), nb, kw)
    one = dev(np.ones(m, dtype=np.float32))
    z = []
    for xb, wpart in ((vb, w[:k]), (nb, w[k:])):
        wb = torch.zeros((m, kw), dtype=torch.int64, device="cuda")
        B.pack_weights_i8(ctx, dev(wpart), k, m, m, wb, kw)
        zf = torch.empty((n, m), dtype=torch.float32, device="cuda")
        B.bgemm(ctx, xb, n, kw, k, kw, wb, m, kw, B.EPI_SCALE_F32, None, one, zf, m)   # BMM.BBF
        z.append(zf)
    ob = torch.zeros((n, mw), dtype=torch.int64, device="cuda")
    B.add(ctx, z[0], False, m, z[1], False, m, n, m, B.EPI_THRESH_BITS,
          dev(t_mm.astype(np.float32)), ob, mw)
    torch.cuda.synchronize()
    assert np.array_equal(words_np(ob), orc.to_words(want))
    adj.close()


def test_add_rejects_bad_arguments(B, ctx):
    f = torch.zeros((4, 70), dtype=torch.float32, device="cuda")
    w = torch.zeros((4, 2), dtype=torch.int64, device="cuda")
    for args, code in (
            ((f, False, 69, f, False, 70, 4, 70, B.EPI_SCALE_F32, None, f, 70), B.ERR_INVALID_ARG),
            ((f, False, 70, w, True, 1, 4, 70, B.EPI_SCALE_F32, None, f, 70), B.ERR_INVALID_ARG),
            ((f, False, 70, f, False, 70, 4, 70, B.EPI_THRESH_BITS, None, w, 2), B.ERR_INVALID_ARG),
            ((f, False, 70, f, False, 70, 4, 70, B.EPI_RAW_I32, None, f, 70), B.ERR_INVALID_ARG),
            ((f, False, 70, f, False, 70, 4, 0, B.EPI_SCALE_F32, None, f, 70), B.ERR_INVALID_ARG),
            ((f, False, 70, None, False, 70, 4, 70, B.EPI_SCALE_F32, None, f, 70), B.ERR_INVALID_ARG),
            ((f, False, 70, w.data_ptr() + 4, True, 2, 4, 70, B.EPI_SCALE_F32, None, f, 70),
             B.ERR_ALIGNMENT)):
        with pytest.raises(B.BitgnnError) as e:
            B.add(ctx, *args)
        assert e.value.code == code, args
    B.add(ctx, None, False, 70, None, False, 70, 0, 70, B.EPI_SCALE_F32, None, None, 70)  # n = 0


# ------------------------------------------------------------------ whole models
def _run_model(B, ctx, wl):
    adj = B.adj_build(ctx, dev(wl.src), dev(wl.dst), len(wl.src), wl.n, wl.adj_flags)
    model = B.BinaryGNN(ctx, wl.model, adj, wl.dims, wl.layers)
    x = dev(wl.x).to(torch.float32)
    logits = model.forward(x)
    torch.cuda.synchronize()
    return adj, model, logits.cpu().numpy()


def _check_model(B, ctx, wl):
    adj, model, logits = _run_model(B, ctx, wl)
    rp, col = orc.adjacency(wl.src, wl.dst, wl.n, wl.adj_flags)
    assert adj.nnz == rp[-1]
    ref, hidden = orc.forward(wl.model, rp, col, orc.bin_f32(wl.x.astype(np.float32)),
                              wl.layers, return_hidden=True)
    # hidden activations: packed words bit-exact (buffer of layer l+1 = output of layer l)
    for l, h in enumerate(hidden):
        kw = (h.shape[1] + 63) // 64
        got = words_np(model.act[l + 1])[:, :kw]
        assert np.array_equal(got, orc.to_words(h)), f"hidden layer {l}"
    assert rel_close(logits, ref), "logits"
    adj.close()


@pytest.mark.parametrize("cfg,kw", [
    (1, {}), (1, {"zero_thresholds": True}), (2, {"n": 1 << 13}), (3, {"n": 20000}),
    (4, {"n": 6000, "mean_deg": 120.0}), (5, {"n": 50000, "mean_deg": 20.0})])
def test_model_small(B, ctx, tuned, cfg, kw):
    _check_model(B, ctx, W.make_workload(cfg, **kw))


@pytest.mark.parametrize("n,e,K,M", [(300, 4000, 7, 3), (2000, 90000, 64, 41),
                                     (5000, 200000, 128, 41), (3000, 150000, 100, 130),
                                     (1500, 40000, 129, 7), (2000, 60000, 300, 41),
                                     (1000, 30000, 512, 70)])
def test_gcn_out_layer_both_orders(B, ctx, tuned, n, e, K, M):
    """The output layer may aggregate first and transform second: same integers."""
    adj, rp, col, r = _graph(B, ctx, n, e, SYM_LOOPS, n + K + M, hubs=1)
    v = W.pm1(r, (n, K))
    w = W.pm1(r, (K, M))
    alpha = r.uniform(0.5, 1.5, M).astype(np.float32)
    ref = orc.gcn_out_layer(rp, col, v, w, alpha)
    kw = (K + 63) // 64
    tmp = torch.zeros((n, M), dtype=torch.int32, device="cuda")
    out = torch.zeros((n, M + 2), dtype=torch.float32, device="cuda")
    B.gcn_out_layer(ctx, adj, _pack_host(v), kw, K, kw, _pack_host(np.ascontiguousarray(w.T)), M,
                    kw, dev(alpha), tmp, out, M + 2)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert rel_close(got[:, :M], ref)
    assert np.all(got[:, M:] == 0)
    # alpha = 1: logits are the exact integers
    one = np.ones(M, dtype=np.float32)
    B.gcn_out_layer(ctx, adj, _pack_host(v), kw, K, kw, _pack_host(np.ascontiguousarray(w.T)), M,
                    kw, dev(one), tmp, out, M + 2)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy()[:, :M], orc.gcn_out_layer(rp, col, v, w, one))
    adj.close()


@pytest.mark.parametrize("n,e,K,M,kind", [
    (120, 500, 33, 5, "sparse"),          # max degree < 2^7: one 7-bit digit
    (20001, 30000, 128, 41, "star"),      # a row of 20,001: three digits
    (2100000, 0, 96, 3, "star")])         # a row of 2.1 million: four digits
def test_gcn_out_layer_digit_counts(B, ctx, n, e, K, M, kind):
    """The fused output layer splits neighbour counts into base-128 digits: cover every
    digit count (the random graphs above have two)."""
    r = np.random.default_rng(n + K)
    src, dst = W.random_graph(r, n, e) if e else (np.zeros(0, np.int32), np.zeros(0, np.int32))
    if kind == "star":
        src = np.concatenate([src, np.zeros(n - 1, dtype=np.int32)])
        dst = np.concatenate([dst, np.arange(1, n, dtype=np.int32)])
    B.ctx_set_tuning(ctx, 8192, 256, 0)   # blocked path whatever the density
    try:
        adj = B.adj_build(ctx, dev(src), dev(dst), len(src), n, SYM_LOOPS)
    finally:
        B.ctx_set_tuning(ctx, *TUNINGS["default"])
    rp, col = orc.adjacency(src, dst, n, SYM_LOOPS)
    assert adj.blocked_info()["parts"] > 0
    if kind == "star":
        assert adj.max_degree == n
    else:
        assert adj.max_degree < 128
    v = W.pm1(r, (n, K))
    w = W.pm1(r, (K, M))
    one = np.ones(M, dtype=np.float32)
    kw = (K + 63) // 64
    tmp = torch.zeros((n, M), dtype=torch.int32, device="cuda")
    out = torch.zeros((n, M), dtype=torch.float32, device="cuda")
    B.gcn_out_layer(ctx, adj, _pack_host(v), kw, K, kw, _pack_host(np.ascontiguousarray(w.T)), M,
                    kw, dev(one), tmp, out, M)
    torch.cuda.synchronize()
    ref = orc.gcn_out_layer(rp, col, v, w, one)
    got = out.cpu().numpy()
    if adj.max_degree * K < (1 << 24):    # integers below 2^24 are exact in float32
        assert np.array_equal(got, ref)
    else:
        assert rel_close(got, ref)
    adj.close()


@pytest.mark.parametrize("n,e,K,M", [(300, 2500, 70, 40), (4000, 60000, 128, 128),
                                     (2500, 30000, 200, 65)])
def test_weighted_layers(B, ctx, n, e, K, M):
    """GCN layer with the symmetrically normalised adjacency and GraphSAGE layer with the
    mean aggregator, against the oracle's compositions (same float32 steps)."""
    adj, rp, col, r = _graph(B, ctx, n, e, SYM_LOOPS, n + K + M)
    deg = np.maximum(orc.degrees(rp), 1).astype(np.float64)
    dinv, mean = (deg ** -0.5).astype(np.float32), (1.0 / deg).astype(np.float32)
    v = W.pm1(r, (n, K))
    kw, mw = (K + 63) // 64, (M + 63) // 64
    # GCN: K -> M
    w = W.pm1(r, (K, M))
    t_mm = r.integers(-4, 5, M).astype(np.int32)
    tau = r.uniform(-0.3, 0.3, M).astype(np.float32)
    tmp = torch.zeros((n, mw), dtype=torch.int64, device="cuda")
    out = torch.zeros((n, mw), dtype=torch.int64, device="cuda")
    B.gcn_layer_weighted(ctx, adj, _pack_host(v), kw, K, kw, _pack_host(np.ascontiguousarray(w.T)),
                         M, kw, dev(t_mm), dev(dinv), dev(dinv), dev(tau), tmp, out, mw)
    torch.cuda.synchronize()
    want = orc.gcn_hidden_layer_norm(rp, col, v, w, t_mm, dinv, dinv, tau)
    assert np.array_equal(words_np(out), orc.to_words(want))
    # SAGE mean: [self | nb] (2K) -> M
    w2 = W.pm1(r, (2 * K, M))
    tau_k = r.uniform(-0.3, 0.3, K).astype(np.float32)
    cat = np.zeros((n, 2 * kw), dtype=np.uint64)
    cat[:, :kw] = orc.to_words(v)
    cat_d = dev(cat.view(np.int64))
    wt = np.ascontiguousarray(w2.T)
    wb = dev(np.concatenate([orc.to_words(wt[:, :K]), orc.to_words(wt[:, K:])], axis=1)
             .view(np.int64))
    out2 = torch.zeros((n, mw), dtype=torch.int64, device="cuda")
    B.sage_layer_weighted(ctx, adj, cat_d, K, wb, M, 2 * kw, dev(mean), None, dev(tau_k),
                          dev(t_mm), out2, mw)
    torch.cuda.synchronize()
    want2 = orc.sage_hidden_layer_mean(rp, col, v, w2, mean, tau_k, t_mm)
    assert np.array_equal(words_np(out2), orc.to_words(want2))
    # normalised 2-layer GCN end to end: hidden layer above, then the weighted output layer
    classes = 7
    w3 = W.pm1(r, (M, classes))
    alpha = r.uniform(0.5, 1.5, classes).astype(np.float32)
    tmpf = torch.zeros((n, classes), dtype=torch.float32, device="cuda")
    logits = torch.zeros((n, classes), dtype=torch.float32, device="cuda")
    B.gcn_out_layer_weighted(ctx, adj, out, mw, M, mw, _pack_host(np.ascontiguousarray(w3.T)),
                             classes, mw, dev(alpha), dev(dinv), dev(dinv), tmpf, logits, classes)
    torch.cuda.synchronize()
    want3 = orc.gcn_out_layer_norm(rp, col, want, w3, alpha, dinv, dinv)
    got3 = logits.cpu().numpy()
    # same steps on both sides; a last-bit difference in alpha * Z would still stay within
    # the rounding bound of the sum, (deg + 4) * 2^-23 * sum|terms|
    zabs = np.abs(orc.scale(orc.bmm(want, w3), alpha)).astype(np.float64)
    mag = orc.spmm_weighted(rp, col, zabs, dinv, dinv)
    assert np.all(np.abs(got3.astype(np.float64) - want3) <=
                  (orc.degrees(rp)[:, None] + 4) * 2.0 ** -23 * mag + 1e-30)
    adj.close()


@pytest.mark.parametrize("n,e,K,M,classes", [(300, 2500, 70, 40, 7), (4000, 60000, 128, 128, 41),
                                             (3000, 20000, 1433, 64, 7),
                                             (60, 300, 33000, 20, 3)])   # K > 32767: float rows
def test_full_precision_aggregation_model(B, ctx, n, e, K, M, classes):
    """The "Ours (full)" recipe end to end: BMM.FBF + BSpMM.FBB on float features, then
    BMM.BBF + BSpMM.FBF, over the symmetrically normalised adjacency; and the hidden layer
    on packed input.  Bits exact, logits within the float32 bound of the float64 sum."""
    adj, rp, col, r = _graph(B, ctx, n, e, SYM_LOOPS, 900 + n)
    x = r.standard_normal((n, K)).astype(np.float32)
    v0 = orc.bin_f32(x)
    w1, w2 = W.pm1(r, (K, M)), W.pm1(r, (M, classes))
    a1 = r.uniform(0.5, 1.5, size=M).astype(np.float32)
    a2 = r.uniform(0.5, 1.5, size=classes).astype(np.float32)
    dinv = (orc.degrees(rp).astype(np.float64) ** -0.5).astype(np.float32)
    tau = (r.standard_normal(M) * 2).astype(np.float32)
    want_h = orc.gcn_hidden_layer_full(rp, col, v0, w1, a1, dinv, dinv, tau)
    want_logits = orc.gcn_out_layer_norm(rp, col, want_h, w2, a2, dinv, dinv)

    kw, mw = (K + 63) // 64, (M + 63) // 64
    w1b = torch.zeros((M, kw), dtype=torch.int64, device="cuda")
    B.pack_weights_i8(ctx, dev(w1), K, M, M, w1b, kw)
    w2b = torch.zeros((classes, mw), dtype=torch.int64, device="cuda")
    B.pack_weights_i8(ctx, dev(w2), M, classes, classes, w2b, mw)
    tmp = torch.empty((n, M), dtype=torch.float32, device="cuda")
    h = torch.zeros((n, mw), dtype=torch.int64, device="cuda")
    dv = dev(dinv)
    B.gcn_layer_full_f32(ctx, adj, dev(x), K, K, None, w1b, M, kw, dev(a1), dv, dv, dev(tau), tmp,
                         h, mw)
    tmp2 = torch.empty((n, classes), dtype=torch.float32, device="cuda")
    logits = torch.empty((n, classes), dtype=torch.float32, device="cuda")
    B.gcn_out_layer_weighted(ctx, adj, h, mw, M, mw, w2b, classes, mw, dev(a2), dv, dv, tmp2,
                             logits, classes)
    torch.cuda.synchronize()
    assert np.array_equal(words_np(h), orc.to_words(want_h))
    assert np.array_equal(logits.cpu().numpy().view(np.uint32), want_logits.view(np.uint32))
    # the same hidden layer from packed input (BMM.BBF + BSpMM.FBB)
    xb = dev(orc.to_words(v0).view(np.int64))
    h2 = torch.zeros((n, mw + 1), dtype=torch.int64, device="cuda")
    B.gcn_layer_full(ctx, adj, xb, kw, K, kw, w1b, M, kw, dev(a1), dv, dv, dev(tau), tmp, h2,
                     mw + 1)
    torch.cuda.synchronize()
    assert np.array_equal(words_np(h2)[:, :mw], orc.to_words(want_h))
    with pytest.raises(B.BitgnnError) as e:
        B.gcn_layer_full(ctx, adj, xb, kw, K, kw, w1b, M, kw, None, dv, dv, dev(tau), tmp, h2,
                         mw + 1)
    assert e.value.code == B.ERR_INVALID_ARG
    adj.close()


def test_forward_ops_equals_forward(B, ctx):
    for cfg, kw in ((4, {"n": 6000, "mean_deg": 120.0}), (3, {"n": 20000})):
        wl = W.make_workload(cfg, **kw)
        adj = B.adj_build(ctx, dev(wl.src), dev(wl.dst), len(wl.src), wl.n, wl.adj_flags)
        model = B.BinaryGNN(ctx, wl.model, adj, wl.dims, wl.layers)
        x = dev(wl.x).to(torch.float32)
        a = model.forward(x).clone()
        b = model.forward_ops(x).clone()
        torch.cuda.synchronize()
        assert torch.equal(a, b)
        adj.close()



# ------------------------------------------------------------------ boundary: no allocation
@pytest.mark.parametrize("tuning", ["default", "blocked-small", "csr-only"])
def test_layer_calls_capture_into_a_hip_graph_on_a_fresh_context(B, tuning):
    """Compute calls only enqueue: the first aggregation ever issued on a context may be
    recorded into a HIP graph (nothing allocates or synchronizes under capture), and every
    replay gives the oracle's bits and logits."""
    c = B.Context(0)
    B.ctx_set_tuning(c, *TUNINGS[tuning])
    adj, rp, col, r = _graph(B, c, 6000, 90000, SYM_LOOPS, 4711, hubs=1)
    dims = [200, 128, 41]
    layers = W.model_params(r, "gcn", dims)
    x = W.pm1(r, (6000, dims[0])).astype(np.float32)
    model = B.BinaryGNN(c, "gcn", adj, dims, layers)         # set-up: reserves the workspace
    ref, hidden = orc.forward("gcn", rp, col, orc.bin_f32(x), layers, return_hidden=True)
    xd = dev(x)
    torch.cuda.synchronize()
    before = B.ctx_workspace(c)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        model.forward(xd)                                    # first aggregation: under capture
    assert B.ctx_workspace(c) == before
    for rep in range(3):
        model.act[1].zero_()
        model.logits.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(words_np(model.act[1])[:, :2], orc.to_words(hidden[0])), rep
        assert rel_close(model.logits.cpu().numpy(), ref), rep
        eager = model.forward(xd)                            # eager work between the replays
        torch.cuda.synchronize()
        assert rel_close(eager.cpu().numpy(), ref)
    del graph
    adj.close()
    c.close()


def test_compute_calls_report_a_workspace_that_is_too_small(B):
    """A call that needs more workspace than was reserved fails with ERR_WORKSPACE instead of
    allocating; after bitgnn_ctx_reserve it runs and is right."""
    c = B.Context(0)
    B.ctx_set_tuning(c, *TUNINGS["blocked-small"])
    n, K, M = 500, 64, 9000                                  # 9,000 classes: 1.2 MB of weights
    adj, rp, col, r = _graph(B, c, n, 4000, SYM_LOOPS, 321)
    v = W.pm1(r, (n, K))
    w = W.pm1(r, (K, M))
    alpha = r.uniform(0.5, 1.5, M).astype(np.float32)
    need = B.adj_workspace_bytes(c, adj, K, M)
    assert need > B.ctx_workspace(c)
    tmp = torch.zeros((n, M), dtype=torch.int32, device="cuda")
    out = torch.zeros((n, M), dtype=torch.float32, device="cuda")
    args = (c, adj, _pack_host(v), 1, K, 1, _pack_host(np.ascontiguousarray(w.T)), M, 1,
            dev(alpha), tmp, out, M)
    with pytest.raises(B.BitgnnError) as e:
        B.gcn_out_layer(*args)
    assert e.value.code == B.ERR_WORKSPACE and "bitgnn_ctx_reserve" in str(e.value)
    B.ctx_reserve(c, need)
    assert B.ctx_workspace(c) >= need
    B.gcn_out_layer(*args)
    torch.cuda.synchronize()
    y = orc.spmm_i64(rp, col, orc.bmm(v, w))
    assert rel_close(out.cpu().numpy(), orc.scale(y, alpha))
    adj.close()
    c.close()

# ------------------------------------------------------------------ whole model, one launch
def _fused_case(B, ctx, n, e, dims, flags, seed, hubs=0, real_features=True):
    """A two-layer GCN on a seeded graph through bitgnn_gcn2_fused and through the oracle."""
    adj, rp, col, r = _graph(B, ctx, n, e, flags, seed, hubs)
    layers = W.model_params(r, "gcn", list(dims))
    if real_features:
        x = r.standard_normal((n, dims[0])).astype(np.float32)
        x[r.random((n, dims[0])) < 0.05] = 0.0          # exact zeros binarize to +1
    else:
        x = W.pm1(r, (n, dims[0]), 0.013).astype(np.float32)
    model = B.BinaryGNN(ctx, "gcn", adj, list(dims), layers)
    return adj, rp, col, layers, x, model


def _check_fused(B, model, rp, col, layers, x):
    xd = dev(x)
    assert model.fused_applies
    logits = model.forward_fused(xd)
    torch.cuda.synchronize()
    assert int(model.fused_status.item()) == 0, "a grid barrier wait was abandoned"
    v0 = orc.bin_f32(x)
    ref, hidden = orc.forward("gcn", rp, col, v0, layers, return_hidden=True)
    c1 = hidden[0].shape[1]
    mw = (c1 + 63) // 64
    h = orc.rebin(orc.bmm(v0, layers[0].w), layers[0].t_mm)
    assert np.array_equal(words_np(model.tmp_bits)[:, :mw], orc.to_words(h)), "BMM bits"
    assert np.array_equal(words_np(model.act[1])[:, :mw], orc.to_words(hidden[0])), "hidden bits"
    assert rel_close(logits.cpu().numpy(), ref), "logits"
    return logits.clone(), model.act[1].clone()


@pytest.mark.parametrize("n,e,dims,flags,hubs", [
    (1, 0, (1, 1, 1), W.ADJ_ADD_SELF_LOOPS, 0),
    (5, 6, (70, 64, 7), W.ADJ_SYMMETRIZE, 0),                  # isolated nodes: degree 0 rows
    (300, 1500, (1433, 64, 7), SYM_LOOPS, 0),
    (1000, 5000, (65, 65, 64), SYM_LOOPS, 0),                  # two tiles, ragged; 64 classes
    (2000, 9000, (600, 128, 41), SYM_LOOPS, 1),                # a row of ~1000 neighbours
    (4097, 30000, (129, 256, 10), SYM_LOOPS, 0),               # four tiles
    (3000, 12000, (512, 200, 3), W.ADJ_SYMMETRIZE, 0),         # ragged four tiles
    (20000, 90000, (500, 64, 3), SYM_LOOPS, 0),                # several rows per wavefront
    (20000, 60000, (100, 100, 5), SYM_LOOPS, 0),               # ... with two tiles
    (18000, 50000, (64, 256, 64), W.ADJ_SYMMETRIZE, 0)])       # ... with four tiles
def test_gcn2_fused_matches_oracle_and_layer_calls(B, ctx, n, e, dims, flags, hubs):
    adj, rp, col, layers, x, model = _fused_case(B, ctx, n, e, dims, flags, 500 + n, hubs)
    assert adj.max_degree <= B.FUSED_MAX_DEGREE
    fused_logits, fused_h = _check_fused(B, model, rp, col, layers, x)
    # the un-fused layer calls on the same buffers: identical bits and logits
    model.act[1].zero_()
    model.logits.zero_()
    plain = model.forward(dev(x))
    torch.cuda.synchronize()
    assert torch.equal(model.act[1], fused_h)
    assert torch.equal(plain, fused_logits)
    # again, after other work went through the context: the barrier counter carries on
    model.act[1].zero_()
    model.logits.zero_()
    again = model.forward_fused(dev(x))
    torch.cuda.synchronize()
    assert int(model.fused_status.item()) == 0
    assert torch.equal(model.act[1], fused_h) and torch.equal(again, fused_logits)
    adj.close()


def test_gcn2_fused_config1_full_size(B, ctx):
    wl = W.make_workload(1)
    adj = B.adj_build(ctx, dev(wl.src), dev(wl.dst), len(wl.src), wl.n, wl.adj_flags)
    rp, col = orc.adjacency(wl.src, wl.dst, wl.n, wl.adj_flags)
    model = B.BinaryGNN(ctx, "gcn", adj, wl.dims, wl.layers)
    _check_fused(B, model, rp, col, wl.layers, wl.x.astype(np.float32))
    adj.close()


def test_gcn2_fused_abandoned_wait_is_reported_and_recovered_from(B, ctx):
    """Failure path of the grid barrier, forced from the host: with a bound of one poll the
    workgroups that arrive early give up.  Every workgroup must still exit, the status word
    must say so, and the next call (default bound) must be right: the arrival counter stays
    in step because a workgroup that gave up still arrives at the later barriers."""
    adj, rp, col, layers, x, model = _fused_case(B, ctx, 20000, 90000, (500, 64, 3), SYM_LOOPS,
                                                 4242)
    want_logits, want_h = _check_fused(B, model, rp, col, layers, x)
    B.ctx_set_fused_spin_limit(ctx, 1)
    try:
        model.forward_fused(dev(x))
        torch.cuda.synchronize()
    finally:
        B.ctx_set_fused_spin_limit(ctx, 1 << 22)
    gave_up = int(model.fused_status.item())
    assert gave_up >= 1, "no wait was abandoned with a bound of one poll"
    model.act[1].zero_()
    model.logits.zero_()
    again = model.forward_fused(dev(x))
    torch.cuda.synchronize()
    assert int(model.fused_status.item()) == gave_up          # sticky, nothing new
    assert torch.equal(again, want_logits) and torch.equal(model.act[1], want_h)
    with pytest.raises(B.BitgnnError):
        B.ctx_set_fused_spin_limit(ctx, 0)
    adj.close()


def test_gcn2_fused_replays_from_a_hip_graph(B, ctx):
    """The one-launch model recorded into a HIP graph: every replay, with eager work and
    synchronizations between the replays, gives the eager result."""
    adj, rp, col, layers, x, model = _fused_case(B, ctx, 2708, 5300, (1433, 64, 7), SYM_LOOPS, 99,
                                                 real_features=False)
    want_logits, want_h = _check_fused(B, model, rp, col, layers, x)
    xd = dev(x)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        model.forward_fused(xd)
    for rep in range(4):
        model.act[1].zero_()
        model.logits.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert int(model.fused_status.item()) == 0
        assert torch.equal(model.logits, want_logits), f"replay {rep}"
        assert torch.equal(model.act[1], want_h), f"replay {rep}"
        eager = model.forward(xd) if rep % 2 else model.forward_fused(xd)   # eager work between
        torch.cuda.synchronize()
        assert torch.equal(eager, want_logits)
    del graph
    adj.close()


def test_gcn2_fused_rejects_what_it_cannot_run(B, ctx):
    """Outside its range the call fails before launching, naming the limits."""
    adj, rp, col, layers, x, model = _fused_case(B, ctx, 3000, 9000, (64, 64, 7), SYM_LOOPS, 77,
                                                 hubs=2)
    assert adj.max_degree > B.FUSED_MAX_DEGREE and not model.fused_applies
    with pytest.raises(B.BitgnnError) as e:
        model.forward_fused(dev(x))
    assert e.value.code == B.ERR_RANGE and "degree <= 1024" in str(e.value)
    adj.close()
    adj, rp, col, layers, x, model = _fused_case(B, ctx, 500, 2000, (64, 300, 7), SYM_LOOPS, 78)
    with pytest.raises(B.BitgnnError) as e:
        model.forward_fused(dev(x))
    assert e.value.code == B.ERR_RANGE
    p0, p1 = model.params
    h1 = model.act[1]
    bad = lambda **kw: B.gcn2_fused(**{**dict(
        ctx=ctx, adj=adj, x=dev(x), K0=64, ldx=64, w1bits=p0["wb"], C1=300,
        w1_stride=p0["wb"].stride(0), T_mm=p0["t_mm"], T_agg=p0["t_agg"], w2bits=p1["wb"], M=7,
        w2_stride=p1["wb"].stride(0), alpha=p1["alpha"], tmp_bits=model.tmp_bits, h_bits=h1,
        h_stride=h1.stride(0), logits=model.logits, ldo=7), **kw})
    for kw, code in ((dict(ldx=63), B.ERR_INVALID_ARG), (dict(h_stride=4), B.ERR_INVALID_ARG),
                     (dict(ldo=6), B.ERR_INVALID_ARG), (dict(alpha=None), B.ERR_INVALID_ARG),
                     (dict(M=0), B.ERR_INVALID_ARG),
                     (dict(logits=model.logits.data_ptr() + 2), B.ERR_ALIGNMENT)):
        with pytest.raises(B.BitgnnError) as e:
            bad(**kw)
        assert e.value.code == code, kw
    adj.close()


@pytest.mark.parametrize("cfg", [2, 3])
def test_model_full_size(B, ctx, cfg):
    _check_model(B, ctx, W.make_workload(cfg))


@pytest.mark.parametrize("cfg,kw", [(2, {"n": 1 << 13}), (3, {"n": 20000}),
                                    (4, {"n": 6000, "mean_deg": 120.0})])
def test_model_replayed_from_a_hip_graph(B, ctx, cfg, kw):
    """BinaryGNN.capture: the layer calls of a whole model recorded once, replayed on new
    features with the program's own eager work and synchronizations between the replays;
    every replay gives the oracle's logits and the eager run's bits."""
    wl = W.make_workload(cfg, **kw)
    src, dst = dev(wl.src), dev(wl.dst)
    adj = B.adj_build(ctx, src, dst, len(wl.src), wl.n, wl.adj_flags)
    model = B.BinaryGNN(ctx, wl.model, adj, wl.dims, wl.layers)
    rp, col = orc.adjacency(wl.src, wl.dst, wl.n, wl.adj_flags)
    x = dev(wl.x.astype(np.float32))
    g = model.capture(x)
    r = np.random.default_rng(cfg)
    for rep in range(3):
        xs = (wl.x * (1.0 if rep == 0 else -1.0) +
              (0.0 if rep < 2 else r.normal(0, 1, wl.x.shape))).astype(np.float32)
        x.copy_(dev(xs))                        # new contents at the captured address
        model.logits.fill_(-7.0)
        g.replay()
        torch.cuda.synchronize()
        got = model.logits.cpu().numpy().copy()
        ref = orc.forward(wl.model, rp, col, orc.bin_f32(xs), wl.layers)
        assert rel_close(got, ref), f"replay {rep}"
        eager = model.forward(x).cpu().numpy()  # eager work between the replays
        assert np.array_equal(got, eager), f"replay {rep} against the eager run"
    adj.close()
