"""Seeded synthetic graphs and feature matrices (torch, any device).

The public datasets the paper measures on are not available here and are not
reproduced; these generators only imitate their node counts, edge counts and
degree shape.  Output is always CSR with int64 rowptr, int32 colidx ascending
within a row, float32 val, plus a dense float32 feature matrix.

Input generation only: none of the sampled-SpMM method's arithmetic is here.
"""
from __future__ import annotations

import math

import torch

from . import rng


def _csr_from_keys(keys: torch.Tensor, n: int):
    """Sorted unique keys row*n+col -> (rowptr int64, colidx int32)."""
    row = torch.div(keys, n, rounding_mode="floor")
    col = (keys - row * n).to(torch.int32)
    counts = torch.bincount(row, minlength=n)
    rowptr = torch.zeros(n + 1, dtype=torch.int64, device=keys.device)
    torch.cumsum(counts, 0, out=rowptr[1:])
    return rowptr, col


def _finish_keys(keys: torch.Tensor, n: int, self_loops: bool, relabel_seed):
    """Drop or add the diagonal, relabel nodes, sort and de-duplicate."""
    row = torch.div(keys, n, rounding_mode="floor")
    col = keys - row * n
    keep = row != col
    row, col = row[keep], col[keep]
    if relabel_seed is not None:
        perm = rng.permutation(relabel_seed, 77, n, keys.device)
        row, col = perm[row], perm[col]
    keys = row * n + col
    if self_loops:
        diag = torch.arange(n, dtype=torch.int64, device=keys.device) * (n + 1)
        keys = torch.cat([keys, diag])
    return torch.unique(keys, sorted=True)


def powerlaw_weights(n: int, gamma: float, mean_degree: float, device) -> torch.Tensor:
    """Expected degrees w_i ~ (i + i0)^(-1/(gamma-1)) with mean `mean_degree`;
    i0 is the smallest shift for which max w <= sqrt(sum w) (the Chung-Lu
    condition that keeps edge probabilities below one)."""
    alpha = 1.0 / (gamma - 1.0)
    idx = torch.arange(n, dtype=torch.float64, device=device)
    total = n * mean_degree
    cap = math.sqrt(total)

    def weights(i0: float) -> torch.Tensor:
        w = (idx + i0) ** (-alpha)
        return w * (total / w.sum())

    lo, hi = 1e-3, float(n)
    if float(weights(lo)[0]) <= cap:
        return weights(lo)
    for _ in range(60):
        mid = math.sqrt(lo * hi)
        if float(weights(mid)[0]) > cap:
            lo = mid
        else:
            hi = mid
    return weights(hi)


def lognormal_weights(n: int, mean_degree: float, sigma: float, lo: float, hi: float,
                      seed: int, device) -> torch.Tensor:
    """Expected degrees exp(mu + sigma z), mean `mean_degree` before clipping."""
    mu = math.log(mean_degree) - 0.5 * sigma * sigma
    z = rng.normal(seed, 5, n, device)
    return torch.exp(mu + sigma * z).clamp_(lo, hi)


def chung_lu(weights: torch.Tensor, seed: int, self_loops: bool, relabel: bool):
    """Undirected Chung-Lu wiring: sum(w)/2 endpoint pairs, each endpoint drawn
    with probability proportional to its weight; symmetrised, de-duplicated."""
    device = weights.device
    n = weights.numel()
    m = int(round(float(weights.sum()) / 2.0))
    # Integer cumulative weights: a floating-point prefix sum on the GPU is not reproducible
    # from run to run (its partial sums combine in timing-dependent order); an int64 one is exact.
    wq = torch.clamp((weights * (2.0 ** 40 / float(weights.max()))).to(torch.int64), min=1)
    cdf = torch.cumsum(wq, 0)
    total = int(cdf[-1])
    chunks = []
    step = 1 << 24

    def draw(stream, k, s):
        u = (rng.uniform(seed, stream, k, device, start=s) * float(total)).to(torch.int64).clamp_(max=total - 1)
        return torch.searchsorted(cdf, u, right=True).clamp_(max=n - 1)

    for s in range(0, m, step):
        k = min(step, m - s)
        src = draw(1, k, s)
        dst = draw(2, k, s)
        chunks.append(src * n + dst)
        chunks.append(dst * n + src)
    keys = torch.cat(chunks) if chunks else torch.empty(0, dtype=torch.int64, device=device)
    del chunks
    keys = _finish_keys(keys, n, self_loops, seed if relabel else None)
    return _csr_from_keys(keys, n)


def rmat(scale: int, n_edges: int, a: float, b: float, c: float, seed: int,
         self_loops: bool, relabel: bool, device):
    """Directed R-MAT: every edge picks one quadrant per bit level."""
    n = 1 << scale
    chunks = []
    step = 1 << 24
    for s in range(0, n_edges, step):
        k = min(step, n_edges - s)
        src = torch.zeros(k, dtype=torch.int64, device=device)
        dst = torch.zeros(k, dtype=torch.int64, device=device)
        for level in range(scale):
            u = rng.uniform(seed, 10 + level, k, device, start=s)
            src_bit = (u >= a + b).to(torch.int64)
            dst_bit = (((u >= a) & (u < a + b)) | (u >= a + b + c)).to(torch.int64)
            src = (src << 1) | src_bit
            dst = (dst << 1) | dst_bit
        chunks.append(src * n + dst)
    keys = torch.cat(chunks)
    del chunks
    keys = _finish_keys(keys, n, self_loops, seed if relabel else None)
    return _csr_from_keys(keys, n)


def edge_values(rowptr: torch.Tensor, colidx: torch.Tensor, norm: str) -> torch.Tensor:
    """float32 edge weights.  'sym': 1/sqrt(d_r d_c) (GCN); 'row': 1/d_r
    (GraphSAGE-mean / row-normalised unit weights).  d = stored entries per
    row; computed in float64, rounded once."""
    n = rowptr.numel() - 1
    deg = (rowptr[1:] - rowptr[:-1]).to(torch.float64)
    row = torch.repeat_interleave(torch.arange(n, device=rowptr.device), rowptr[1:] - rowptr[:-1])
    if norm == "sym":
        v = 1.0 / torch.sqrt(deg[row] * deg[colidx.long()].clamp_(min=1.0))
    elif norm == "row":
        v = 1.0 / deg[row]
    else:
        raise ValueError(norm)
    return v.to(torch.float32)


def features(n: int, F: int, dist: str, seed: int, device, ld: int | None = None) -> torch.Tensor:
    """Dense n x F float32; 'normal' = N(0,1), 'uniform' = U(-1,1).  The result
    is a view of an n x ld buffer (ld >= F) when ld is given."""
    ld = F if ld is None else ld
    buf = torch.zeros((n, ld), dtype=torch.float32, device=device)
    rows_per = max(1, (1 << 24) // max(F, 1))
    for r0 in range(0, n, rows_per):
        r1 = min(n, r0 + rows_per)
        cnt = (r1 - r0) * F
        if dist == "normal":
            x = _normal_at(seed, r0 * F, cnt, device)
        elif dist == "uniform":
            x = rng.uniform(seed, 40, cnt, device, start=r0 * F) * 2.0 - 1.0
        else:
            raise ValueError(dist)
        buf[r0:r1, :F] = x.to(torch.float32).view(r1 - r0, F)
    return buf[:, :F]


def _normal_at(seed: int, start: int, cnt: int, device) -> torch.Tensor:
    u1 = 1.0 - rng.uniform(seed, 41, cnt, device, start=start)
    u2 = rng.uniform(seed, 42, cnt, device, start=start)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
