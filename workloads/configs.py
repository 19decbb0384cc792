"""The benchmark configurations as seeded synthetic inputs.

Each full-size entry imitates the shape (node count, edge count, degree
distribution, normalisation, feature width) of one workload; the `*_small`
entries are the same recipes shrunk so that a CPU-only test finishes in
seconds.  `make(name, device)` returns a dict of torch tensors on `device`.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import torch

from . import graphs

Q_PER_TENSOR, Q_PER_COLUMN, Q_PER_ROW = 0, 1, 2
Q_AFFINE_FLOOR_U8, Q_SYMMETRIC_RNE_I8 = 0, 1


@dataclass(frozen=True)
class Workload:
    name: str
    kind: str                  # 'powerlaw' | 'lognormal' | 'rmat'
    n: int
    mean_degree: float
    gamma: float = 0.0         # powerlaw exponent
    sigma: float = 1.0         # lognormal shape
    max_degree: float = 0.0    # lognormal clip
    rmat_scale: int = 0
    rmat_edges: int = 0
    self_loops: bool = True
    norm: str = "sym"          # 'sym' | 'row'
    F: int = 128
    x_dist: str = "normal"
    widths: tuple = (64,)
    q_scheme: int = Q_SYMMETRIC_RNE_I8
    q_granularity: int = Q_PER_COLUMN
    seed: int = 0
    extra: dict = field(default_factory=dict)


WORKLOADS = {w.name: w for w in [
    # configs[0]: tiny power-law graph, fp32 sampled SpMM only
    Workload("tiny", "powerlaw", 4096, 4.0, gamma=2.1, norm="sym", F=64, widths=(32,), seed=0),
    # configs[1]: citation-network-shaped
    Workload("arxiv_like", "powerlaw", 170_000, 7.0, gamma=2.2, norm="sym", F=128,
             widths=(32, 64), q_granularity=Q_PER_COLUMN, seed=1),
    # configs[2]: dense social-network-shaped, log-normal degrees
    Workload("reddit_like", "lognormal", 233_000, 490.0, sigma=1.0, max_degree=20_000.0,
             norm="sym", F=256, widths=(64, 128, 256), q_granularity=Q_PER_COLUMN, seed=2),
    # configs[3]: co-purchase-shaped, the largest graph
    Workload("products_like", "powerlaw", 2_450_000, 50.0, gamma=2.0, self_loops=False,
             norm="row", F=128, widths=(64,), q_granularity=Q_PER_ROW, seed=3),
    # configs[4]: R-MAT width sweep
    Workload("rmat20", "rmat", 1 << 20, 64.0, rmat_scale=20, rmat_edges=1 << 26, norm="row",
             F=256, x_dist="uniform", widths=(16, 32, 64, 128, 256),
             q_granularity=Q_PER_COLUMN, seed=4),
    # beyond the five benchmark configurations: a citation-graph shape two orders of magnitude larger
    # (111 M nodes, ~1.66 G stored entries), to exercise 64-bit indexing and the 288 GB of one MI355X
    Workload("papers_like", "powerlaw", 111_000_000, 14.0, gamma=2.2, norm="row", F=128,
             widths=(32,), q_granularity=Q_PER_ROW, seed=9),
    # shrunk recipes for CPU-only tests and quick GPU parity
    Workload("arxiv_small", "powerlaw", 6_000, 7.0, gamma=2.2, norm="sym", F=128,
             widths=(32, 64), q_granularity=Q_PER_COLUMN, seed=11),
    Workload("reddit_small", "lognormal", 3_000, 300.0, sigma=1.0, max_degree=2_500.0,
             norm="sym", F=256, widths=(64, 128, 256), q_granularity=Q_PER_COLUMN, seed=12),
    Workload("products_small", "powerlaw", 20_000, 50.0, gamma=2.0, self_loops=False,
             norm="row", F=128, widths=(64,), q_granularity=Q_PER_ROW, seed=13),
    Workload("rmat12", "rmat", 1 << 12, 64.0, rmat_scale=12, rmat_edges=1 << 18, norm="row",
             F=256, x_dist="uniform", widths=(16, 32, 64, 128, 256),
             q_granularity=Q_PER_COLUMN, seed=14),
]}


def make_graph(w: Workload, device):
    dev = torch.device(device)
    if w.kind == "powerlaw":
        wt = graphs.powerlaw_weights(w.n, w.gamma, w.mean_degree, dev)
        rowptr, colidx = graphs.chung_lu(wt, w.seed, w.self_loops, relabel=True)
    elif w.kind == "lognormal":
        wt = graphs.lognormal_weights(w.n, w.mean_degree, w.sigma, 1.0, w.max_degree, w.seed, dev)
        rowptr, colidx = graphs.chung_lu(wt, w.seed, w.self_loops, relabel=False)
    elif w.kind == "rmat":
        rowptr, colidx = graphs.rmat(w.rmat_scale, w.rmat_edges, 0.57, 0.19, 0.19, w.seed,
                                     w.self_loops, relabel=True, device=dev)
    else:
        raise ValueError(w.kind)
    val = graphs.edge_values(rowptr, colidx, w.norm)
    return rowptr, colidx, val


def make(name: str, device="cpu", ldx: int | None = None):
    """Build workload `name`: dict(rowptr, colidx, val, X, n, nnz, F, workload)."""
    w = WORKLOADS[name]
    rowptr, colidx, val = make_graph(w, device)
    X = graphs.features(w.n, w.F, w.x_dist, w.seed + 1000, torch.device(device), ld=ldx)
    return {"workload": w, "n": w.n, "nnz": int(colidx.numel()), "F": w.F,
            "rowptr": rowptr, "colidx": colidx, "val": val, "X": X}
