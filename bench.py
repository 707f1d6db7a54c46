#!/usr/bin/env python3
"""Benchmark of the binary-GNN hot path on one MI355X.

A step is one full-graph inference of the configured model: bit-pack of the
float features, then every layer (XNOR-popcount BGEMM, bit-SpMM with fused
threshold/re-pack, integer aggregation + scale for the logits), with all inputs
and the prebuilt adjacency already resident in HBM.  The adjacency build and the
weight packing are done once before the timed region (they are offline steps in
the paper) and their time is reported separately.

Prints ONE JSON line: `value` = bit operations of a step (N K M per BMM, nnz C per
aggregation) / step time; `kernels` = per library call, from HIP events on the launch
stream; `roofline` = the dominant kernel's algorithmic bytes / its own launch time against
the HBM peak, with the HBM traffic the profiler's counters report; `cpu_baseline` = the CPU
oracle timed on the host cores on the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0                       # MI355X HBM3E
VALU_PEAK_TLOPS = 256 * 64 * 2.4e9 / 1e12   # 256 CUs x 64 lanes x 2.4 GHz, 32-bit lane-ops
MFMA_I8_PEAK_TOPS = 5000.0                  # dense int8 matrix cores


def source_stamp():
    """Identifies the aggregation kernels and the format builder the counter summaries under
    profiles/ were taken with: counters of other code are not this run's."""
    import hashlib
    h = hashlib.sha1()
    for f in ("bspmm.hip", "adj_blocked.hip", "bgemm.hip", "bgemm_mfma.hip", "pack.hip"):
        h.update(open(os.path.join(ROOT, "paper_2305_02522_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:12]


def load_counters(cfg, stored_ids):
    """profiles/bench_cfg<N>_counters.txt: per kernel, figures derived from rocprofv3 --pmc runs
    of this command (HBM bytes per launch, VALU busy, ...).  Returns {} when the file was
    taken with other kernel sources or another aggregation format."""
    path = os.path.join(ROOT, "profiles", f"bench_cfg{cfg}_counters.txt")
    if not os.path.exists(path):
        return {}
    out, ok = {}, False
    for line in open(path):
        t = line.split()
        if line.startswith("# stamp:"):
            kv = dict(x.split("=") for x in t[2:])
            ok = kv.get("src") == source_stamp() and int(kv.get("stored_ids", -1)) == stored_ids
        elif t and t[0] == "kernel" and len(t) >= 2:
            # t[1] = kernel name with its template arguments, e.g. bspmm_blk_kernel<8,16>
            short, _, targs = t[1].partition("<")
            out.setdefault(short, {})["<" + targs if targs else ""] = {
                t[i]: float(t[i + 1]) for i in range(2, len(t) - 1, 2)}
    return out if ok else {}


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def op_models(wl, nnz, blocked, fused=False, bgemm_kernel=None):
    """Per-op work (bit-ops) and algorithmic bytes / lane-ops, keyed like forward_ops labels.
    Index bytes of an aggregation = min(bytes of the format the kernel actually streams,
    CSR at 4 B per non-zero), so a padded format earns no bandwidth credit.
    bgemm_kernel(n, kwords, M) -> "valu" | "mfma": the kernel the library launches for a
    packed-operand BMM; it sets the op's roofline (vector lane-ops, or int8 matrix-core
    operations on the bits widened to bytes: 2 N K M)."""
    n = wl.n
    bgemm_kernel = bgemm_kernel or (lambda rows, kwords, m: "valu")

    def bgemm_op(k_bits, kwords, m, bytes_):
        op = dict(work=n * k_bits * m, bytes=bytes_)
        if bgemm_kernel(n, kwords, m) == "mfma":
            op.update(bound="mfma", mfma_ops=2 * n * kwords * 64 * m, kernel="bgemm_mfma_kernel")
        else:
            op.update(bound="alu", lane_ops=2 * n * m * 2 * kwords, kernel="bgemm_kernel")
        return op

    w64 = lambda k: (k + 63) // 64
    idx_bytes = 4 * nnz + 4 * (n + 1)
    if blocked["parts"]:
        fmt = 2 * blocked["stored_ids"] + 4 * (blocked["tiles"] + 2 * blocked["slices"]) \
            + 4 * (n + 1) + 4 * blocked["parts"]
        idx_bytes = min(idx_bytes, fmt)
    ops = {}
    k0 = wl.dims[0]
    nl = len(wl.layers)
    if fused:
        # the whole two-layer GCN in one launch: features and weights once, the CSR arrays
        # for each of the two aggregations, both bit matrices written and read, the logits
        c1, m = wl.dims[1], wl.dims[2]
        ops["gcn2_fused"] = dict(
            work=n * k0 * c1 + nnz * c1 + n * c1 * m + nnz * m,
            bytes=4 * n * k0 + 8 * w64(k0) * c1 + 2 * (4 * nnz + 8 * (n + 1))
            + 4 * 8 * n * w64(c1) + 8 * w64(c1) * m + 4 * n * m, bound="hbm")
        return ops
    fused_first = wl.model == "gcn" and nl > 1      # float features feed the first product
    if not fused_first:
        ops["pack_f32"] = dict(work=0, bytes=4 * n * k0 + 8 * n * w64(k0), bound="hbm")
    for l in range(nl):
        k_in, m = wl.dims[l], wl.dims[l + 1]
        last = l == nl - 1
        if wl.model == "gcn":
            kw = w64(k_in)
            out_b = 4 * n * m if last else 8 * n * w64(m)
            if last:
                # transform + aggregate + scale in one driver call
                ops[f"L{l}.out_layer"] = dict(work=n * k_in * m + nnz * m,
                                              bytes=idx_bytes + 8 * n * kw + 8 * kw * m + 4 * n
                                              + 4 * n * m, bound="hbm")
            elif l == 0:
                ops[f"L{l}.bgemm_f32"] = dict(work=n * k_in * m,
                                              bytes=4 * n * k_in + 8 * kw * m + out_b,
                                              lane_ops=2 * n * m * ((k_in + 31) // 32),
                                              bound="hbm")
            else:
                ops[f"L{l}.bgemm"] = bgemm_op(k_in, kw, m, 8 * kw * (n + m) + out_b)
            if not last:
                ops[f"L{l}.bspmm"] = dict(work=nnz * m,
                                          bytes=idx_bytes + 16 * n * w64(m) + 4 * n + 4 * m,
                                          bound="hbm")
        else:
            kw = w64(k_in)
            ops[f"L{l}.bspmm"] = dict(work=nnz * k_in,
                                      bytes=idx_bytes + 16 * n * kw + 4 * n + 4 * k_in,
                                      bound="hbm")
            out_b = 4 * n * m if last else 8 * n * w64(m)
            ops[f"L{l}.bgemm"] = bgemm_op(2 * k_in, 2 * kw, m, 16 * kw * (n + m) + out_b)
    # the same ops priced with CSR's index bytes, whatever format is stored: a measure that
    # does not move when the stored format shrinks or grows
    for lab, op in ops.items():
        if lab.endswith(".bspmm") or lab.endswith(".out_layer"):
            op["bytes_csr"] = op["bytes"] - idx_bytes + 4 * nnz + 4 * (n + 1)
    return ops


def cpu_baseline(wl, rows):
    """The oracle, as it stands, on the first `rows` nodes of every step of the model
    (inputs of the right shape and distribution; hidden activations are seeded +-1
    draws, not GPU results).  Returns (bit-ops per second, seconds, threads)."""
    import numpy as np
    from oracle import oracle as orc
    from paper_2305_02522_amd import workloads as W
    rng = np.random.default_rng(7)
    rp, col = orc.adjacency(wl.src, wl.dst, wl.n, wl.adj_flags)
    rows = min(rows, wl.n)
    deg_rows = int(rp[rows] - rp[0])
    work, secs = 0, 0.0
    x = wl.x[:rows].astype(np.float32)
    t = time.perf_counter()
    v = orc.bin_f32(x)
    secs += time.perf_counter() - t
    nl = len(wl.layers)
    for l, p in enumerate(wl.layers):
        k_in, m = wl.dims[l], wl.dims[l + 1]
        last = l == nl - 1
        # untimed: seeded stand-ins for the activations of ALL nodes that the
        # aggregation of the sampled rows gathers from
        if wl.model == "gcn" and last:
            gathered = rng.integers(-k_in, k_in + 1, size=(wl.n, m)).astype(np.int64)
        else:
            gathered = W.pm1(rng, (wl.n, m if wl.model == "gcn" else k_in))
        t = time.perf_counter()
        if wl.model == "gcn":
            z = orc.bmm(v, p.w)
            if last:
                orc.scale(orc.spmm_i64(rp, col, gathered, (0, rows)), p.alpha)
            else:
                orc.rebin(z, p.t_mm)
                v = orc.rebin(orc.spmm_pm1(rp, col, gathered, (0, rows)), p.t_agg)
            work += rows * k_in * m + deg_rows * m
        else:
            nb = orc.rebin(orc.spmm_pm1(rp, col, gathered, (0, rows)), p.t_agg)
            z = orc.bmm(orc.concat(gathered[:rows], nb), p.w)
            if last:
                orc.scale(z, p.alpha)
            else:
                v = orc.rebin(z, p.t_mm)
            work += deg_rows * k_in + rows * 2 * k_in * m
        secs += time.perf_counter() - t
    return work / secs, secs, orc.max_threads()


def bench_spmm_f32(args, np, torch, B, ctx, adj, wl):
    """D^-1/2 A D^-1/2 X on the workload's graph, X float32 with the first hidden width
    (full-precision aggregation) and X as packed bits (weighted binary aggregation): one
    JSON line.  Bytes a launch must move: the column ids and the factor of every stored
    non-zero once, every activation row once, the output once; the gathers of rows that
    follow are served by the caches or re-read."""
    n, nnz, C = wl.n, adj.nnz, int(wl.dims[1])
    r = np.random.default_rng(7)
    import ctypes
    deg = torch.empty(n, dtype=torch.int32, device="cuda")
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
    assert hip.hipMemcpy(deg.data_ptr(), adj.csr_pointers()[2], 4 * n, 3) == 0
    dinv = (torch.clamp(deg.to(torch.float64), min=1.0) ** -0.5).to(torch.float32)
    xf = torch.as_tensor(r.standard_normal((n, C)).astype(np.float32), device="cuda")
    xb = torch.as_tensor(r.integers(-2**62, 2**62, size=(n, (C + 63) // 64)), device="cuda")
    out = torch.empty((n, C), dtype=torch.float32, device="cuda")
    res = {}
    for name, x, bits, ldx in (("f32", xf, 0, C), ("bits", xb, 1, (C + 63) // 64)):
        for _ in range(max(1, args.warmup)):
            B.spmm_f32(ctx, adj, x, bits, C, ldx, dinv, dinv, B.EPI_SCALE_F32, None, out, C)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            B.spmm_f32(ctx, adj, x, bits, C, ldx, dinv, dinv, B.EPI_SCALE_F32, None, out, C)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        row_bytes = 8 * ((C + 63) // 64) if bits else 4 * C
        alg = nnz * 8 + n * (row_bytes + 4 * C + 12)
        res[name] = {"ms": round(ms, 4), "gather_bytes": nnz * row_bytes,
                     "roofline": {"bound": "hbm", "achieved": round(alg / ms / 1e6, 1),
                                  "peak": 8000.0, "unit": "GB/s",
                                  "frac": round(alg / ms / 1e6 / 8000.0, 4), "traffic": None}}
        log(f"spmm_f32 {name}: {ms:.3f} ms, gathers {nnz * row_bytes / ms / 1e6:.0f} GB/s")
    print(json.dumps({
        "metric": "weighted aggregation D^-1/2 A D^-1/2 X (G edge-channel MAC/s), float activations",
        "value": round(nnz * C / res["f32"]["ms"] / 1e6, 1), "unit": "G edge-channel MAC/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["f32"]["ms"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"cfg{args.config} {wl.name}", "N": n, "nnz": nnz, "C": C},
        "roofline": res["f32"]["roofline"], "bits_activations": res["bits"]}))


def bench_gcn_full(args, np, torch, B, ctx, adj, wl):
    """The two-layer GCN of the workload in the full-precision-aggregation recipe (products
    binarized, aggregation in float32 over D^-1/2 A D^-1/2): BMM.FBF + BSpMM.FBB, then
    BMM.BBF + BSpMM.FBF.  One JSON line; the roofline record is the first aggregation's
    (float rows of the hidden width), the dominant kernel."""
    assert wl.model == "gcn" and len(wl.layers) == 2, "--op gcn_full needs a two-layer GCN config"
    n, nnz = wl.n, adj.nnz
    k0, c1, m = (int(d) for d in wl.dims)
    r = np.random.default_rng(7)
    import ctypes
    deg = torch.empty(n, dtype=torch.int32, device="cuda")
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
    assert hip.hipMemcpy(deg.data_ptr(), adj.csr_pointers()[2], 4 * n, 3) == 0
    dinv = (torch.clamp(deg.to(torch.float64), min=1.0) ** -0.5).to(torch.float32)
    kw, mw = (k0 + 63) // 64, (c1 + 63) // 64
    w1b = torch.zeros((c1, kw), dtype=torch.int64, device="cuda")
    w2b = torch.zeros((m, mw), dtype=torch.int64, device="cuda")
    B.pack_weights_i8(ctx, torch.as_tensor(wl.layers[0].w, device="cuda"), k0, c1, c1, w1b, kw)
    B.pack_weights_i8(ctx, torch.as_tensor(wl.layers[1].w, device="cuda"), c1, m, m, w2b, mw)
    a1 = torch.as_tensor(r.uniform(0.5, 1.5, size=c1).astype(np.float32), device="cuda")
    a2 = torch.as_tensor(wl.layers[1].alpha, device="cuda")
    tau = torch.as_tensor(r.standard_normal(c1).astype(np.float32), device="cuda")
    x = torch.as_tensor(wl.x, device="cuda").to(torch.float32)
    tmp1 = torch.empty((n, c1), dtype=torch.float32, device="cuda")
    tmp2 = torch.empty((n, m), dtype=torch.float32, device="cuda")
    h = torch.zeros((n, mw), dtype=torch.int64, device="cuda")
    logits = torch.empty((n, m), dtype=torch.float32, device="cuda")
    marks = []

    def step(timed):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        ev[0].record()
        B.gcn_layer_full_f32(ctx, adj, x, k0, k0, None, w1b, c1, kw, a1, dinv, dinv, tau, tmp1, h,
                             mw)
        ev[1].record()
        B.gcn_out_layer_weighted(ctx, adj, h, mw, c1, mw, w2b, m, mw, a2, dinv, dinv, tmp2,
                                 logits, m)
        ev[2].record()
        if timed:
            marks.append(ev)

    for _ in range(max(1, args.warmup)):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    l1 = float(np.mean([e[0].elapsed_time(e[1]) for e in marks]))
    l2 = float(np.mean([e[1].elapsed_time(e[2]) for e in marks]))
    work = n * k0 * c1 + nnz * c1 + n * c1 * m + nnz * m
    alg = nnz * 8 + n * (4 * c1 + 8 * mw + 12)          # ids + factors, float rows in, bits out
    log(f"gcn_full: {ms:.3f} ms per model (layer 1 {l1:.3f} ms, layer 2 {l2:.3f} ms)")
    print(json.dumps({
        "metric": "binary GNN, full-precision aggregation recipe (G edge-channel + node-feature "
                  "MAC/s) + full-graph inference ms, 1 GPU",
        "value": round(work / ms / 1e6, 1), "unit": "G MAC/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32 aggregation / u64 bit-packed products",
        "data": "synthetic",
        "config": {"workload": f"cfg{args.config} {wl.name}: 2-layer GCN, full-precision "
                               f"aggregation, N={n}, nnz={nnz}, dims={wl.dims}",
                   "layer_ms": [round(l1, 4), round(l2, 4)]},
        "roofline": {"kernel": "spmm_f32_kernel", "op": "L0 aggregation (float rows)",
                     "bound": "hbm", "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": None, "traffic": None, "alg_MB": round(alg / 1e6, 2),
                     "note": "bench.py --op spmm_f32 times this kernel alone"}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, help="workload 1..5 (default 4: the "
                    "232,965-node Reddit-shaped 2-layer GCN the roofline target is stated on)")
    ap.add_argument("--cpu-rows", type=int, default=1 << 30,
                    help="rows of the workload the CPU oracle is timed on (default: all)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true",
                    help="skip the leg that replays the step from a captured HIP graph")
    ap.add_argument("--cold-steps", type=int, default=5,
                    help="steps of the cache-flushed leg (1.25 GB swept through the caches "
                    "before each; reported beside the steady-state numbers; 0 = skip)")
    ap.add_argument("--unfused", action="store_true",
                    help="time the layer calls even where the one-launch kernel applies "
                    "(two-layer GCN on a small graph, e.g. --config 1)")
    ap.add_argument("--op", choices=["model", "spmm_f32", "gcn_full"], default="model",
                    help="model: the binary GNN forward pass (the headline metric); spmm_f32: "
                    "the symmetric-normalised full-precision aggregation on the same graph; "
                    "gcn_full: the two-layer GCN with full-precision aggregation")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                 "use --gpus 1")

    import numpy as np
    import torch
    from paper_2305_02522_amd import binding as B
    from paper_2305_02522_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    t0 = time.perf_counter()
    wl = W.make_workload(args.config)
    log(f"workload cfg{args.config} {wl.name}: N={wl.n} raw pairs={len(wl.src)} "
        f"({time.perf_counter() - t0:.1f}s)")
    ctx = B.Context(0)
    src = torch.as_tensor(wl.src, device="cuda")
    dst = torch.as_tensor(wl.dst, device="cuda")
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    adj = B.adj_build(ctx, src, dst, len(wl.src), wl.n, wl.adj_flags)
    build_ms = (time.perf_counter() - t1) * 1e3
    del src, dst
    log(f"adjacency: nnz={adj.nnz} max_degree={adj.max_degree} build {build_ms:.1f} ms "
        f"blocked={adj.blocked_info()}")
    if args.op == "spmm_f32":
        return bench_spmm_f32(args, np, torch, B, ctx, adj, wl)
    if args.op == "gcn_full":
        return bench_gcn_full(args, np, torch, B, ctx, adj, wl)
    model = B.BinaryGNN(ctx, wl.model, adj, wl.dims, wl.layers)
    x = torch.as_tensor(wl.x, device="cuda").to(torch.float32)
    torch.cuda.synchronize()

    # one plain device copy of known size: calibrates the rocprofv3 FETCH_SIZE / WRITE_SIZE
    # counters when this command runs under the profiler (outside the timed region)
    calib = torch.empty_like(x)
    calib.copy_(x)
    log(f"calibration copy: {x.numel() * 4} bytes read and written")
    del calib

    fused = model.fused_applies and not args.unfused
    if fused:
        log("small graph: the whole model runs as ONE launch (bitgnn_gcn2_fused)")

    def run_step(mark=None):
        if not fused:
            return model.forward_ops(x, mark)
        if mark:
            mark("gcn2_fused")
        model.forward_fused(x)
        if mark:
            mark(None)

    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()

    # timed region: K steps, one HIP event before every library call (torch's current
    # stream is the stream the library launches on); the library itself brackets its
    # main aggregation kernel with HIP events on the same stream
    labels, events = [], []
    first_step = [True]

    def mark(label):
        ev = torch.cuda.Event(enable_timing=True)
        ev.record()
        events[-1].append(ev)
        if first_step[0]:
            labels.append(label)
            if label is None:
                first_step[0] = False

    B.ctx_kernel_timing(ctx, True)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        events.append([])
        run_step(mark)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_start) * 1e3
    agg_ms = B.ctx_kernel_times(ctx)
    B.ctx_kernel_timing(ctx, False)

    per_op = {lab: [] for lab in labels if lab}
    step_ms = []
    for evs in events:
        step_ms.append(evs[0].elapsed_time(evs[-1]))
        for i, lab in enumerate(labels[:-1]):
            per_op[lab].append(evs[i].elapsed_time(evs[i + 1]))
    ms_per_step = wall_ms / args.steps
    blocked = adj.blocked_info()
    if fused:
        assert int(model.fused_status.item()) == 0, "a grid barrier wait was abandoned"
    def bgemm_kernel(rows, kwords, m):
        return "mfma" if B.ctx_bgemm_kernel(ctx, rows, kwords, m) == B.BGEMM_MFMA else "valu"
    models = op_models(wl, adj.nnz, blocked, fused, bgemm_kernel)
    total_work = sum(m["work"] for m in models.values())
    value = total_work / (ms_per_step * 1e-3) / 1e9

    # aggregation launches of one step, in call order (a 128-channel window each)
    agg_labels = []
    for lab in [l for l in labels if l]:
        if lab.endswith(".bspmm"):
            c = wl.dims[int(lab[1:lab.index(".")]) + (1 if wl.model == "gcn" else 0)]
            agg_labels += [lab] * ((c + 127) // 128 if blocked["parts"] else 1)
        elif lab.endswith(".out_layer") and blocked["parts"] and wl.dims[-2] <= 128:
            agg_labels.append(lab)
    agg_kernel_ms = {}
    csr_labels = [l for l in labels if l and l.endswith(".bspmm")]
    took_blocked = bool(blocked["parts"]) and bool(agg_labels) and \
        len(agg_ms) == len(agg_labels) * args.steps
    if not took_blocked and csr_labels and len(agg_ms) == len(csr_labels) * args.steps:
        agg_labels = csr_labels          # the library chose the CSR kernel: one launch per call
    if agg_labels and len(agg_ms) == len(agg_labels) * args.steps:
        for i, lab in enumerate(agg_labels):
            agg_kernel_ms.setdefault(lab, []).extend(agg_ms[i::len(agg_labels)])

    counters = load_counters(args.config, blocked["stored_ids"])

    def fractions(m, ms, launches=1.0):
        """Roofline fractions of an op (or of one of its launches) that took `ms`."""
        f = dict(hbm_frac=round(m["bytes"] / launches / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4))
        if "lane_ops" in m:
            f["valu_frac"] = round(m["lane_ops"] / (ms * 1e-3) / 1e12 / VALU_PEAK_TLOPS, 4)
        if "mfma_ops" in m:
            f["mfma_i8_frac"] = round(m["mfma_ops"] / (ms * 1e-3) / 1e12 / MFMA_I8_PEAK_TOPS, 4)
        for name, v in f.items():
            assert v <= 1.0, f"{name} = {v} > 1: the op model does not describe the kernel that ran"
        return f

    def kernel_name(lab):
        kind = lab.split(".")[-1]
        if kind == "bgemm":
            return models[lab]["kernel"]
        return {"bspmm": "bspmm_blk_kernel" if took_blocked else "bspmm_kernel",
                "out_layer": "bspmm_blk_kernel" if lab in agg_kernel_ms else "spmm_i32_kernel",
                "bgemm_f32": "bgemm_f32_kernel", "gcn2_fused": "gcn2_fused_kernel",
                "pack_f32": "pack_rows4_kernel"}[kind]

    kernels = {}
    for lab, ts in per_op.items():
        avg = float(np.mean(ts))
        m = models[lab]
        k = dict(kernel=kernel_name(lab), avg_us=round(avg * 1e3, 2),
                 min_us=round(float(np.min(ts)) * 1e3, 2), alg_MB=round(m["bytes"] / 1e6, 2),
                 bound=m["bound"], **fractions(m, avg))
        if m["work"]:
            k["Gbit_ops_per_s"] = round(m["work"] / (avg * 1e-3) / 1e9, 1)
        if lab in agg_kernel_ms:      # the aggregation kernel alone (sum over channel windows)
            per_call = len(agg_kernel_ms[lab]) / args.steps
            k["agg_kernel_us"] = round(float(np.mean(agg_kernel_ms[lab])) * per_call * 1e3, 2)
        c = counters.get(k["kernel"])
        if c:                         # from the rocprofv3 --pmc summaries under profiles/
            pick = lambda v: {key: v[key] for key in ("us", "valu_busy", "lds_busy", "mfma_busy",
                                                      "hbm_MB", "l2_hit") if key in v}
            k["counters"] = pick(next(iter(c.values()))) if len(c) == 1 else \
                {targs: pick(v) for targs, v in c.items()}     # one entry per instantiation
        kernels[lab] = k

    # roofline of the dominant kernel: for an aggregation op that is the library-timed
    # aggregation kernel (one launch), for the other ops the op is a single kernel; the
    # whole call (with its permute / merge launches) is reported beside it
    def kernel_time_ms(lab):
        if lab in agg_kernel_ms:
            return float(np.mean(agg_kernel_ms[lab])), len(agg_kernel_ms[lab]) / args.steps
        return float(np.mean(per_op[lab])), 1.0
    dom = max(per_op, key=lambda lab: kernel_time_ms(lab)[0] * kernel_time_ms(lab)[1])
    dm = models[dom]
    davg, launches = kernel_time_ms(dom)
    kname = kernel_name(dom)
    fr = fractions(dm, davg, launches)
    if dm["bound"] == "hbm":
        ach, peak, unit, frac = fr["hbm_frac"] * HBM_PEAK_GBS, HBM_PEAK_GBS, "GB/s", fr["hbm_frac"]
    elif dm["bound"] == "mfma":
        ach, peak, unit, frac = (fr["mfma_i8_frac"] * MFMA_I8_PEAK_TOPS, MFMA_I8_PEAK_TOPS,
                                 "TOP/s", fr["mfma_i8_frac"])
    else:
        ach, peak, unit, frac = (fr["valu_frac"] * VALU_PEAK_TLOPS, round(VALU_PEAK_TLOPS, 2),
                                 "Tlane-op/s", fr["valu_frac"])
    call_avg = float(np.mean(per_op[dom]))
    roofline = dict(kernel=kname, op=dom, bound=dm["bound"], achieved=round(ach, 1), peak=peak,
                    unit=unit, frac=frac, avg_launch_us=round(davg * 1e3, 2),
                    call={"avg_us": round(call_avg * 1e3, 2), **fractions(dm, call_avg)},
                    traffic=None)
    if "bytes_csr" in dm:   # the launch priced at CSR's 4 bytes per non-zero
        roofline["frac_at_csr_bytes"] = round(
            dm["bytes_csr"] / launches / (davg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    c = counters.get(kname)
    if c:       # the instantiation whose duration is closest to this run's launches
        v = min(c.values(), key=lambda v: abs(v.get("us", 0.0) - davg * 1e3))
        roofline["traffic"] = int(v["hbm_MB"] * 1e6)
        roofline["valu_busy"] = v.get("valu_busy")
        roofline["traffic_frac_of_hbm_peak"] = round(
            v["hbm_MB"] * 1e6 / (v["us"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4) if v.get("us") else None

    # HIP-graph leg: the same step captured once and replayed K times (no instrumentation
    # inside): what the launches and the event records of the timed region cost
    graph_leg = None
    if not args.no_graph:
        try:
            logits_ref = model.logits.clone()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                run_step()
            for _ in range(2):
                g.replay()
            torch.cuda.synchronize()
            tg = time.perf_counter()
            for _ in range(args.steps):
                g.replay()
            torch.cuda.synchronize()
            g_ms = (time.perf_counter() - tg) * 1e3 / args.steps
            graph_leg = {"ms_per_step": round(g_ms, 4),
                         "Gbit_edge_ops_per_s": round(total_work / g_ms / 1e6, 1),
                         "logits_equal_eager": bool(torch.equal(logits_ref, model.logits))}
            del g
        except Exception as e:      # capture is an extra: report, do not fail the bench
            graph_leg = {"error": str(e)[:200]}
            torch.cuda.synchronize()

    # cache-flushed leg: the same step with > 1 GB swept through the caches before every
    # step (the 256 MB Infinity Cache and the L2 then hold none of the operands)
    cold = None
    if args.cold_steps > 0:
        sweep = torch.empty(320 * 1024 * 1024, dtype=torch.float32, device="cuda")  # 1.25 GB
        cold_ev = []
        for _ in range(args.cold_steps):
            sweep.add_(1.0)
            events.clear()
            events.append([])
            run_step(mark)
            cold_ev.append(events[-1])
        torch.cuda.synchronize()
        cold_ops = {lab: [] for lab in per_op}
        cold_step = []
        for evs in cold_ev:
            cold_step.append(evs[0].elapsed_time(evs[-1]))
            for i, lab in enumerate(labels[:-1]):
                cold_ops[lab].append(evs[i].elapsed_time(evs[i + 1]))
        cold = {"steps": args.cold_steps, "flush_MB": round(sweep.numel() * 8 / 1e6),
                "ms_per_step": round(float(np.mean(cold_step)), 4),
                "Gbit_edge_ops_per_s": round(total_work / float(np.mean(cold_step)) / 1e6, 1),
                "kernels_avg_us": {lab: round(float(np.mean(v)) * 1e3, 2)
                                   for lab, v in cold_ops.items()}}
        del sweep

    result = {
        "metric": "binary GNN layer throughput (Gbit-edge-ops/s) + full-graph inference ms, 1 GPU",
        "value": round(value, 1), "unit": "Gbit-edge-ops/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u64 bit-packed / int32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"cfg{args.config} {wl.name}: {len(wl.layers)}-layer binary "
                               f"{wl.model.upper()}, N={wl.n}, nnz={adj.nnz}, dims={wl.dims}",
                   "inference_ms_event_median": round(float(np.median(step_ms)), 4),
                   "adj_build_ms": round(build_ms, 1), "bit_ops_per_step": total_work,
                   "aggregation_format": blocked},
        "kernels": kernels, "roofline": roofline,
    }
    if graph_leg:
        result["graph_replay"] = graph_leg
    if cold:
        result["cache_flushed"] = cold
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a row sample ...")
        rate, secs, threads = cpu_baseline(wl, args.cpu_rows)
        result["cpu_baseline"] = {
            "value": round(rate / 1e9, 3), "unit": "Gbit-edge-ops/s", "cores": threads,
            "kind": "oracle",
            "sample": f"every step of the model on the first {min(args.cpu_rows, wl.n)} nodes "
                      f"({secs:.1f} s of oracle time)"}
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
