"""Seeded synthetic workloads shaped like the graphs of the paper's Table 2.

This module only draws inputs: graphs (edge lists), +-1 features, +-1 weights,
integer thresholds and float scales.  It contains none of the method's
arithmetic (no packing, no dot products, no aggregation), so that it can feed
both the CPU oracle and the HIP library without the two sharing any code.

The real datasets (Cora, Flickr, Reddit, ...; paper Table 2) are not available
here; these generators stand in for them with the same node counts, feature
widths, class counts and mean degrees:

    cfg 1  Cora-shaped     stochastic block model, 7 blocks      2-layer GCN
    cfg 2  R-MAT scale 17  edge factor 16, (a,b,c)=(.57,.19,.19)  3-layer GCN
    cfg 3  Flickr-shaped   Chung-Lu power law, mean degree 10    2-layer SAGE
    cfg 4  Reddit-shaped   Chung-Lu power law, mean degree 492   2-layer GCN
    cfg 5  products-shaped Chung-Lu power law, mean degree 50    3-layer SAGE

Every edge list is the raw list of drawn pairs: it may contain duplicates
(and, for R-MAT, loops); the adjacency is the *set* of pairs after
symmetrisation, which is what both the oracle and the library build from it.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

BASE_SEED = 23050252

ADJ_SYMMETRIZE = 1
ADJ_ADD_SELF_LOOPS = 2


@dataclass
class LayerParams:
    """Parameters of one binary layer.

    w      int8 [K_total, M], entries +-1 (for SAGE K_total = 2*K_in: rows
           0..K_in-1 multiply the node's own bits, rows K_in.. the aggregated
           neighbour bits)
    t_mm   int32 [M]   threshold applied to the BGEMM accumulator (hidden layers)
    t_agg  int32 [C]   threshold applied to the aggregation accumulator
                       (GCN hidden: C = M; SAGE: C = K_in)
    alpha  float32 [M] per-class scale of the last layer, else None
    """
    w: np.ndarray
    t_mm: Optional[np.ndarray]
    t_agg: Optional[np.ndarray]
    alpha: Optional[np.ndarray]


@dataclass
class Workload:
    cfg: int
    name: str
    model: str              # "gcn" | "sage"
    n: int                  # nodes
    src: np.ndarray         # int32 [E] raw drawn pairs
    dst: np.ndarray         # int32 [E]
    adj_flags: int          # ADJ_SYMMETRIZE [| ADJ_ADD_SELF_LOOPS]
    x: np.ndarray           # int8 [N, K0], entries +-1 (cast to f32 for pack_f32)
    dims: List[int]         # [K0, hidden..., classes]
    layers: List[LayerParams] = field(default_factory=list)
    seed: int = 0


# --------------------------------------------------------------------------
# graphs
# --------------------------------------------------------------------------

def sbm_graph(rng: np.random.Generator, n: int, blocks: int, mean_deg: float,
              intra: float = 0.8):
    """Stochastic block model with `blocks` near-equal blocks.

    Each unordered pair inside a block is an edge with probability p_in, across
    blocks with p_out, chosen so a node expects intra*mean_deg neighbours inside
    its block and (1-intra)*mean_deg outside.  Returns unordered pairs (u < v).
    """
    sizes = [n // blocks + (1 if b < n % blocks else 0) for b in range(blocks)]
    start = np.concatenate([[0], np.cumsum(sizes)])
    us, vs = [], []
    for b in range(blocks):
        nb = sizes[b]
        p_in = intra * mean_deg / (nb - 1)
        m = nb * (nb - 1) // 2
        k = rng.binomial(m, p_in)
        # sample k distinct unordered pairs inside the block by rejection
        a = rng.integers(0, nb, size=4 * k + 64)
        c = rng.integers(0, nb, size=4 * k + 64)
        keep = a < c
        key = np.unique(a[keep].astype(np.int64) * nb + c[keep])
        key = rng.permutation(key)[:k]
        us.append(start[b] + key // nb)
        vs.append(start[b] + key % nb)
    # cross-block pairs: draw the total count, then endpoints in different blocks
    block_of = np.repeat(np.arange(blocks), sizes)
    p_out_pairs = 0.0
    for b in range(blocks):
        p_out_pairs += sizes[b] * (1.0 - intra) * mean_deg
    k_out = rng.poisson(p_out_pairs / 2.0)
    a = rng.integers(0, n, size=2 * k_out + 16)
    c = rng.integers(0, n, size=2 * k_out + 16)
    keep = block_of[a] != block_of[c]
    a, c = a[keep][:k_out], c[keep][:k_out]
    us.append(np.minimum(a, c))
    vs.append(np.maximum(a, c))
    u = np.concatenate(us).astype(np.int32)
    v = np.concatenate(vs).astype(np.int32)
    return u, v


def rmat_graph(rng: np.random.Generator, scale: int, edge_factor: int,
               a: float, b: float, c: float):
    """R-MAT: every draw picks one quadrant per bit level with probabilities
    (a, b, c, 1-a-b-c).  Returns the raw directed draws (duplicates and loops
    included)."""
    n = 1 << scale
    m = edge_factor * n
    src = np.zeros(m, dtype=np.int64)
    dst = np.zeros(m, dtype=np.int64)
    for _ in range(scale):
        r = rng.random(m)
        row_bit = r >= (a + b)                       # quadrants c, d
        col_bit = ((r >= a) & (r < a + b)) | (r >= a + b + c)   # quadrants b, d
        src = (src << 1) | row_bit
        dst = (dst << 1) | col_bit
    return src.astype(np.int32), dst.astype(np.int32)


def chung_lu_weights(n: int, mean_deg: float, gamma: float = 2.1,
                     r0: float = 10.0) -> np.ndarray:
    """Expected degrees w_r ~ (r + r0)^(-1/(gamma-1)), capped at sqrt(n*mean_deg)
    and rescaled (bisection on the scale) so that they sum to n*mean_deg."""
    total = float(n) * mean_deg
    cap = np.sqrt(total)
    raw = (np.arange(n, dtype=np.float64) + r0) ** (-1.0 / (gamma - 1.0))
    lo, hi = 0.0, total / raw[-1]
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if np.minimum(cap, mid * raw).sum() < total:
            lo = mid
        else:
            hi = mid
    return np.minimum(cap, hi * raw)


def chung_lu_graph(rng: np.random.Generator, n: int, mean_deg: float,
                   gamma: float = 2.1):
    """Chung-Lu by endpoint sampling: n*mean_deg/2 unordered pairs whose two
    endpoints are drawn independently with probability proportional to the
    expected degree.  Loops are dropped, duplicates are left in."""
    w = chung_lu_weights(n, mean_deg, gamma)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    m = int(round(n * mean_deg / 2.0))
    chunks_u, chunks_v = [], []
    step = 1 << 24
    for lo in range(0, m, step):
        k = min(step, m - lo)
        u = np.searchsorted(cdf, rng.random(k), side="right").astype(np.int32)
        v = np.searchsorted(cdf, rng.random(k), side="right").astype(np.int32)
        np.minimum(u, n - 1, out=u)
        np.minimum(v, n - 1, out=v)
        keep = u != v
        chunks_u.append(u[keep])
        chunks_v.append(v[keep])
    return np.concatenate(chunks_u), np.concatenate(chunks_v)


def relabel(rng: np.random.Generator, n: int, u: np.ndarray, v: np.ndarray):
    """Random vertex relabelling so that a vertex id says nothing about degree."""
    perm = rng.permutation(n).astype(np.int32)
    return perm[u], perm[v]


# --------------------------------------------------------------------------
# features and parameters
# --------------------------------------------------------------------------

def pm1(rng: np.random.Generator, shape, p_plus: float = 0.5) -> np.ndarray:
    """int8 array of +-1 with P(+1) = p_plus."""
    if p_plus == 0.5:
        bits = rng.integers(0, 2, size=shape, dtype=np.int8)
    else:
        bits = (rng.random(shape, dtype=np.float32) < p_plus).astype(np.int8)
    bits *= 2
    bits -= 1
    return bits


def thresholds(rng: np.random.Generator, m: int, zero: bool = False) -> np.ndarray:
    if zero:
        return np.zeros(m, dtype=np.int32)
    return rng.integers(-4, 5, size=m, dtype=np.int32)


def model_params(rng: np.random.Generator, model: str, dims: List[int],
                 zero_thresholds: bool = False) -> List[LayerParams]:
    layers = []
    nl = len(dims) - 1
    for l in range(nl):
        k_in, m = dims[l], dims[l + 1]
        last = l == nl - 1
        k_tot = k_in if model == "gcn" else 2 * k_in
        w = pm1(rng, (k_tot, m))
        if model == "gcn":
            t_mm = None if last else thresholds(rng, m, zero_thresholds)
            t_agg = None if last else thresholds(rng, m, zero_thresholds)
        else:
            t_agg = thresholds(rng, k_in, zero_thresholds)
            t_mm = None if last else thresholds(rng, m, zero_thresholds)
        alpha = rng.uniform(0.5, 1.5, size=m).astype(np.float32) if last else None
        layers.append(LayerParams(w=w, t_mm=t_mm, t_agg=t_agg, alpha=alpha))
    return layers


# --------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------

_SPECS = {
    1: dict(name="cora-shaped-sbm", model="gcn", n=2708, dims=[1433, 64, 7],
            p_plus=0.013, self_loops=True),
    2: dict(name="rmat-s17", model="gcn", n=1 << 17, dims=[512, 256, 256, 40],
            p_plus=0.5, self_loops=True),
    3: dict(name="flickr-shaped-chunglu", model="sage", n=89250,
            dims=[500, 256, 7], p_plus=0.5, self_loops=False, mean_deg=10.0),
    4: dict(name="reddit-shaped-chunglu", model="gcn", n=232965,
            dims=[602, 128, 41], p_plus=0.5, self_loops=True, mean_deg=492.0),
    5: dict(name="products-shaped-chunglu", model="sage", n=2449029,
            dims=[100, 256, 256, 47], p_plus=0.5, self_loops=False,
            mean_deg=50.0),
}


def spec(cfg: int) -> dict:
    return dict(_SPECS[cfg])


def make_workload(cfg: int, n: Optional[int] = None,
                  mean_deg: Optional[float] = None,
                  zero_thresholds: bool = False,
                  seed: Optional[int] = None) -> Workload:
    """Build configuration `cfg` (1..5).  `n` / `mean_deg` shrink it (same
    recipe, fewer nodes or edges) for tests that must finish on a CPU."""
    s = spec(cfg)
    seed = BASE_SEED + 1000 * cfg if seed is None else seed
    rng = np.random.default_rng(np.random.PCG64(seed))
    nn = s["n"] if n is None else int(n)
    if cfg == 1:
        u, v = sbm_graph(rng, nn, 7, 3.9)
        u, v = relabel(rng, nn, u, v)
    elif cfg == 2:
        scale = int(np.log2(nn))
        nn = 1 << scale
        u, v = rmat_graph(rng, scale, 16, 0.57, 0.19, 0.19)
        u, v = relabel(rng, nn, u, v)
    else:
        md = s["mean_deg"] if mean_deg is None else float(mean_deg)
        u, v = chung_lu_graph(rng, nn, md)
        u, v = relabel(rng, nn, u, v)
    flags = ADJ_SYMMETRIZE | (ADJ_ADD_SELF_LOOPS if s["self_loops"] else 0)
    x = pm1(rng, (nn, s["dims"][0]), s["p_plus"])
    layers = model_params(rng, s["model"], s["dims"], zero_thresholds)
    return Workload(cfg=cfg, name=s["name"], model=s["model"], n=nn,
                    src=np.ascontiguousarray(u, dtype=np.int32),
                    dst=np.ascontiguousarray(v, dtype=np.int32),
                    adj_flags=flags, x=x, dims=list(s["dims"]), layers=layers,
                    seed=seed)


def random_graph(rng: np.random.Generator, n: int, e: int):
    """Uniform random directed pairs (duplicates and loops allowed): the
    generic small-case input of the unit tests."""
    return (rng.integers(0, n, size=e, dtype=np.int32),
            rng.integers(0, n, size=e, dtype=np.int32))
