"""The entry point that allocates nothing (bitgnn_bspmm_static): its output must equal
bitgnn_bspmm's, bit for bit, on two calls in a row, the second on a smaller input, on both
aggregation formats; beyond the static array's size it must refuse."""
import numpy as np
import pytest
import torch

from paper_2305_02522_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2305_02522_amd import binding
    return binding


def _dev(a):
    return torch.as_tensor(np.ascontiguousarray(a), device="cuda")


def _case(B, ctx, n, e, C, seed):
    r = np.random.default_rng(seed)
    src, dst = W.random_graph(r, n, e)
    flags = W.ADJ_SYMMETRIZE | W.ADJ_ADD_SELF_LOOPS
    adj = B.adj_build(ctx, _dev(src), _dev(dst), len(src), n, flags)
    cw = (C + 63) // 64
    h = torch.from_numpy(r.integers(-2**63, 2**63 - 1, size=(n, cw), dtype=np.int64)).cuda()
    if C % 64:                                   # pad bits of the input are zero
        h[:, -1] &= (1 << (C % 64)) - 1
    t = _dev(r.integers(-5, 6, size=C).astype(np.int32))
    return adj, h, t, cw


@pytest.mark.parametrize("tuning", [(10208, 255, 8), (10208, 255, 1 << 30), (128, 16, 0)])
def test_static_scratch_entry_point_equals_bspmm(B, tuning):
    ctx = B.Context(0)
    B.ctx_set_tuning(ctx, *tuning)
    for n, e, C, seed in ((30000, 600000, 128, 1), (7000, 50000, 100, 2)):   # second: smaller
        adj, h, t, cw = _case(B, ctx, n, e, C, seed)
        want_bits = torch.full((n, cw), -1, dtype=torch.int64, device="cuda")
        got_bits = torch.full((n, cw), -1, dtype=torch.int64, device="cuda")
        want_raw = torch.full((n, C), 7, dtype=torch.int32, device="cuda")
        got_raw = torch.full((n, C), 7, dtype=torch.int32, device="cuda")
        B.bspmm(ctx, adj, h, C, cw, B.EPI_THRESH_BITS, t, want_bits, cw)
        B.bspmm(ctx, adj, h, C, cw, B.EPI_RAW_I32, None, want_raw, C)
        before = torch.cuda.memory_allocated(), B.ctx_workspace(ctx)
        B.bspmm_static(ctx, adj, h, C, cw, B.EPI_THRESH_BITS, t, got_bits, cw)
        B.bspmm_static(ctx, adj, h, C, cw, B.EPI_RAW_I32, None, got_raw, C)
        torch.cuda.synchronize()
        assert (torch.cuda.memory_allocated(), B.ctx_workspace(ctx)) == before
        assert torch.equal(got_bits, want_bits), (n, "bits")
        assert torch.equal(got_raw, want_raw), (n, "raw")
        adj.close()
    ctx.close()


def test_static_scratch_entry_point_refuses_what_does_not_fit(B):
    ctx = B.Context(0)
    B.ctx_set_tuning(ctx, 8192, 255, 0)          # the column-blocked form, whatever its padding
    n, e, C = 400000, 4000000, 64                # 400 K nodes x 16 B + parts x 128 B > 32 MiB
    adj, h, t, cw = _case(B, ctx, n, e, C, 3)
    assert B.adj_workspace_bytes(ctx, adj, C, 1) > B.STATIC_SCRATCH_BYTES
    out = torch.zeros((n, cw), dtype=torch.int64, device="cuda")
    with pytest.raises(B.BitgnnError) as ex:
        B.bspmm_static(ctx, adj, h, C, cw, B.EPI_THRESH_BITS, t, out, cw)
    assert ex.value.code == B.ERR_UNSUPPORTED and "static array" in str(ex.value)
    B.bspmm(ctx, adj, h, C, cw, B.EPI_THRESH_BITS, t, out, cw)           # the other one runs
    torch.cuda.synchronize()
    adj.close()
    ctx.close()
