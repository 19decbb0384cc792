"""GPU parity at the benchmark's full sizes, in the launch configuration
bench.py times: the plan and the 8-bit codes are compared with the oracle in
full (bit for bit); Y is compared on a seeded sample of rows that the oracle
computes one by one."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

AFF, SYM = 0, 1
N_ROWS_CHECKED = 4000


@pytest.fixture(scope="module")
def G():
    import gpu_common
    assert torch.cuda.is_available(), "these tests need the GPU"
    return gpu_common


def _run(G, name, widths, exact=False, schemes=(SYM,)):
    from workloads import configs
    d = configs.make(name, "cuda")
    w = d["workload"]
    print(f"[{name}] n={d['n']} nnz={d['nnz']} F={d['F']}", flush=True)
    rowptr, col, val = (d[k].cpu().numpy() for k in ("rowptr", "colidx", "val"))
    X = d["X"]
    Xh = X.cpu().numpy()
    rows = np.sort(np.random.default_rng(1).choice(d["n"], size=min(N_ROWS_CHECKED, d["n"]), replace=False))
    # the sample always holds the longest rows too
    rows = np.unique(np.concatenate([rows, np.argsort(np.diff(rowptr))[-8:]])).astype(np.int64)
    q = {s: G.check_quantize(X, s, w.q_granularity) for s in schemes}
    for W in tuple(widths) + ((0,) if exact else ()):
        plan, ref = G.check_plan(d["rowptr"], d["colidx"], d["val"], d["n"], W, 0)
        _, c, g = G.check_f32(plan, ref, X, rows=rows)
        print(f"[{name}] W={W} slots={int(ref[0][-1])} fp32 err comp={c:.2e} glob={g:.2e}", flush=True)
        for s in schemes:
            _, c, g = G.check_q8(plan, ref, q[s][0], q[s][1], s, w.q_granularity, rows=rows)
            print(f"[{name}] W={W} int8 scheme={s} err comp={c:.2e} glob={g:.2e}", flush=True)
        del plan, ref
    # a short-row property that holds at any size: rows with nnz <= W are exact SpMM rows
    return d


def test_arxiv_like(G):
    _run(G, "arxiv_like", (32, 64), schemes=(SYM, AFF))


def test_products_like(G):
    _run(G, "products_like", (64,), schemes=(SYM,))


def test_reddit_like(G):
    _run(G, "reddit_like", (64, 128, 256), exact=True, schemes=(SYM,))


def test_rmat20(G):
    _run(G, "rmat20", (16, 32, 64, 128, 256), schemes=(SYM,))
