"""GPU parity at the full sizes of the two large workloads (the 232,965-node
Reddit-shaped GCN that bench.py times, and the 2,449,029-node products-shaped
GraphSAGE), in the launch configuration bench.py uses (default tuning, the model
runner's forward()).  The oracle computes every layer from its OWN previous layer,
never from a GPU result; hidden activations must match word for word, logits to
1e-5 relative.  The oracle needs tens of seconds per layer on the host cores, so
the big model is checked one layer per test and progress goes to stderr."""
import sys
import time

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2305_02522_amd import workloads as W

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


def say(msg):
    sys.__stderr__.write(f"[full-config] {msg}\n")
    sys.__stderr__.flush()


def dev(a):
    return torch.as_tensor(np.ascontiguousarray(a), device="cuda")


def words_np(t):
    return t.cpu().numpy().view(np.uint64)


def rel_err(got, ref):
    denom = np.maximum(np.abs(ref), 1e-30)
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64)) / denom
    err[got == ref] = 0
    return err.max()


class _Run:
    """One workload: GPU forward once, oracle advanced layer by layer on demand."""

    def __init__(self, cfg):
        from paper_2305_02522_amd import binding as B
        t = time.time()
        self.wl = wl = W.make_workload(cfg)
        say(f"cfg{cfg}: generated N={wl.n} pairs={len(wl.src)} in {time.time() - t:.0f}s")
        self.ctx = B.Context(0)
        self.adj = B.adj_build(self.ctx, dev(wl.src), dev(wl.dst), len(wl.src), wl.n, wl.adj_flags)
        self.model = B.BinaryGNN(self.ctx, wl.model, self.adj, wl.dims, wl.layers)
        self.logits = self.model.forward(dev(wl.x).to(torch.float32)).cpu().numpy()
        torch.cuda.synchronize()
        say(f"cfg{cfg}: GPU forward done, nnz={self.adj.nnz}, blocked={self.adj.blocked_info()}")
        t = time.time()
        self.rp, self.col = orc.adjacency(wl.src, wl.dst, wl.n, wl.adj_flags)
        say(f"cfg{cfg}: oracle adjacency in {time.time() - t:.0f}s")
        self.v = orc.bin_f32(wl.x.astype(np.float32))
        self.done = 0

    def oracle_layer(self, l):
        """Advance the oracle to the output of layer l (layers must be asked in order)."""
        assert l == self.done
        wl, p = self.wl, self.wl.layers[l]
        last = l == len(wl.layers) - 1
        t = time.time()
        if wl.model == "gcn":
            out = orc.gcn_out_layer(self.rp, self.col, self.v, p.w, p.alpha) if last else \
                orc.gcn_hidden_layer(self.rp, self.col, self.v, p.w, p.t_mm, p.t_agg)
        else:
            out = orc.sage_out_layer(self.rp, self.col, self.v, p.w, p.t_agg, p.alpha) if last else \
                orc.sage_hidden_layer(self.rp, self.col, self.v, p.w, p.t_agg, p.t_mm)
        say(f"cfg{wl.cfg}: oracle layer {l} in {time.time() - t:.0f}s")
        self.done += 1
        if not last:
            self.v = out
        return out

    def check_layer(self, l):
        out = self.oracle_layer(l)
        if l == len(self.wl.layers) - 1:
            e = rel_err(self.logits, out)
            assert e <= 1e-5, f"logits max rel err {e}"
        else:
            kw = (out.shape[1] + 63) // 64
            got = words_np(self.model.act[l + 1])[:, :kw]
            ref = np.empty_like(got)
            step = 1 << 18                       # pack the reference in row chunks
            for lo in range(0, out.shape[0], step):
                ref[lo:lo + step] = orc.to_words(out[lo:lo + step])
            assert np.array_equal(got, ref), f"hidden layer {l} differs"


_runs = {}


def _run(cfg):
    if cfg not in _runs:
        _runs.clear()                            # keep one big workload in memory at a time
        _runs[cfg] = _Run(cfg)
    return _runs[cfg]


def test_cfg4_adjacency_and_layer0():
    r = _run(4)
    assert r.adj.nnz == r.rp[-1]
    assert r.adj.max_degree == orc.degrees(r.rp).max()
    assert r.adj.blocked_info()["parts"] > 0     # the LDS-staged path is the one that ran
    r.check_layer(0)


def test_cfg4_logits():
    _run(4).check_layer(1)


def test_cfg4_weighted_aggregation_sampled_rows():
    """The symmetric-normalised aggregation at full size (what `bench.py --op spmm_f32`
    times: float rows and bit rows, C = the first hidden width), on sampled output rows the
    oracle computes one by one: the hub rows, the lowest-degree rows and a random sample."""
    from paper_2305_02522_amd import binding as B
    r = _run(4)
    n, C = r.wl.n, int(r.wl.dims[1])
    deg = orc.degrees(r.rp)
    dinv = (np.maximum(deg, 1).astype(np.float64) ** -0.5).astype(np.float32)
    rng = np.random.default_rng(5)
    xf = rng.standard_normal((n, C)).astype(np.float32)
    v = W.pm1(rng, (n, C))
    order = np.argsort(-deg, kind="stable")
    rows = np.unique(np.concatenate([order[:8], order[-64:], rng.integers(0, n, 600)]))
    tau = rng.uniform(-0.2, 0.2, C).astype(np.float32)
    cw = (C + 63) // 64
    for bits, xh in ((0, xf), (1, v.astype(np.float32))):
        xd = dev(orc.to_words(v).view(np.int64)) if bits else dev(xf)
        out = torch.empty((n, C), dtype=torch.float32, device="cuda")
        ob = torch.empty((n, cw), dtype=torch.int64, device="cuda")
        B.spmm_f32(r.ctx, r.adj, xd, bits, C, cw if bits else C, dev(dinv), dev(dinv),
                   B.EPI_SCALE_F32, None, out, C)
        B.spmm_f32(r.ctx, r.adj, xd, bits, C, cw if bits else C, dev(dinv), dev(dinv),
                   B.EPI_THRESH_BITS, dev(tau), ob, cw)
        torch.cuda.synchronize()
        got, gotb = out.cpu().numpy(), words_np(ob)
        for i in rows:
            want = orc.spmm_weighted_f32(r.rp, r.col, xh, dinv, dinv, rows=(int(i), int(i) + 1))
            assert np.array_equal(got[i:i + 1], want), f"row {i} (degree {deg[i]}) bits={bits}"
            assert np.array_equal(gotb[i:i + 1], orc.to_words(orc.rebin_f32(want, tau)))
    say(f"cfg4: weighted aggregation checked on {len(rows)} rows, degrees up to {deg[rows].max()}")


def test_cfg4_full_precision_aggregation_layer_sampled_rows():
    """The hidden layer of the full-precision-aggregation recipe at full size (what
    `bench.py --op gcn_full` times: float features, BMM kept as integers, aggregated from
    int16 rows with the scale applied inside), on sampled output rows.  The oracle forms
    z = alpha * (bin(x) W) for all nodes in float32 and sums the sampled rows step by step."""
    from paper_2305_02522_amd import binding as B
    r = _run(4)
    wl = r.wl
    n, K, M = wl.n, int(wl.dims[0]), int(wl.dims[1])
    deg = orc.degrees(r.rp)
    dinv = (np.maximum(deg, 1).astype(np.float64) ** -0.5).astype(np.float32)
    rng = np.random.default_rng(6)
    alpha = rng.uniform(0.5, 1.5, M).astype(np.float32)
    tau = rng.uniform(-0.5, 0.5, M).astype(np.float32)
    t = time.time()
    v0 = orc.bin_f32(wl.x.astype(np.float32))
    z = np.empty((n, M), dtype=np.float32)
    step = 1 << 15
    for lo in range(0, n, step):
        z[lo:lo + step] = orc.scale(orc.bmm(v0[lo:lo + step], wl.layers[0].w), alpha)
    say(f"cfg4: oracle scaled product in {time.time() - t:.0f}s")
    kw, mw = (K + 63) // 64, (M + 63) // 64
    wb = torch.zeros((M, kw), dtype=torch.int64, device="cuda")
    B.pack_weights_i8(r.ctx, dev(wl.layers[0].w), K, M, M, wb, kw)
    tmp = torch.empty((n, M), dtype=torch.float32, device="cuda")
    h = torch.zeros((n, mw), dtype=torch.int64, device="cuda")
    B.gcn_layer_full_f32(r.ctx, r.adj, dev(wl.x).to(torch.float32), K, K, None, wb, M, kw,
                         dev(alpha), dev(dinv), dev(dinv), dev(tau), tmp, h, mw)
    torch.cuda.synchronize()
    got = words_np(h)
    order = np.argsort(-deg, kind="stable")
    rows = np.unique(np.concatenate([order[:8], order[-64:], rng.integers(0, n, 600)]))
    for i in rows:
        y = orc.spmm_weighted_f32(r.rp, r.col, z, dinv, dinv, rows=(int(i), int(i) + 1))
        assert np.array_equal(got[i:i + 1], orc.to_words(orc.rebin_f32(y, tau))), \
            f"row {i} (degree {deg[i]})"
    say(f"cfg4: full-precision-aggregation layer checked on {len(rows)} rows")


def test_cfg5_adjacency_and_layer0():
    r = _run(5)
    assert r.adj.nnz == r.rp[-1]
    assert r.adj.max_degree == orc.degrees(r.rp).max()
    r.check_layer(0)


def test_cfg5_layer1():
    _run(5).check_layer(1)


def test_cfg5_logits():
    _run(5).check_layer(2)
    _runs.clear()
