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
    import paper_2503_18427_amd as aes
    q = {s: G.check_quantize(X, s, w.q_granularity) for s in schemes}
    deg = d["rowptr"][1:] - d["rowptr"][:-1]
    Y_exact = None
    for W in ((0,) if exact else ()) + tuple(widths):
        plan, ref = G.check_plan(d["rowptr"], d["colidx"], d["val"], d["n"], W, 0)
        Y, c, g = G.check_f32(plan, ref, X, rows=rows, use_perm=False)        # bench.py's launch configuration
        print(f"[{name}] W={W} slots={int(ref[0][-1])} fp32 err comp={c:.2e} glob={g:.2e}", flush=True)
        # properties that hold at any size, checked on EVERY row: the single-kernel form is
        # bit-identical, and rows that fit (row_nnz <= W) are bit-identical to the unsampled product
        Yf = aes.aes_spmm_fused_f32(d["rowptr"], d["colidx"], d["val"], d["n"], W, X)
        torch.cuda.synchronize()
        assert torch.equal(Yf, Y)
        del Yf
        if W == 0:
            Y_exact = Y
        elif Y_exact is not None:
            short = deg <= W
            assert torch.equal(Y[short], Y_exact[short])
        for s in schemes:
            _, c, g = G.check_q8(plan, ref, q[s][0], q[s][1], s, w.q_granularity, rows=rows, use_perm=False)
            print(f"[{name}] W={W} int8 scheme={s} err comp={c:.2e} glob={g:.2e}", flush=True)
        del plan, ref
    return d


def test_arxiv_like(G):
    _run(G, "arxiv_like", (32, 64), schemes=(SYM, AFF))


def test_products_like(G):
    _run(G, "products_like", (64,), schemes=(SYM,))


def test_reddit_like(G):
    _run(G, "reddit_like", (64, 128, 256), exact=True, schemes=(SYM,))


def test_rmat20(G):
    _run(G, "rmat20", (16, 32, 64, 128, 256), schemes=(SYM,))


def test_entry_indices_beyond_2_31(G):
    """A matrix with 2.6 billion stored entries (48 rows of 54 M): every sampled
    entry index needs 64 bits.  Plan (with source indices) bit-exact against the
    oracle, plan and fused multiplies against the oracle's product."""
    import oracle as orc
    import paper_2503_18427_amd as aes
    n_rows, per_row, n_cols, F, W = 48, 54_000_000, 100_000, 64, 64
    nnz = n_rows * per_row
    assert nnz > 2 ** 31
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    col = torch.randint(0, n_cols, (nnz,), dtype=torch.int32, device="cuda", generator=g)
    val = torch.rand(nnz, device="cuda", generator=g)
    rowptr = torch.arange(0, nnz + 1, per_row, dtype=torch.int64, device="cuda")
    X = torch.randn((n_cols, F), device="cuda", generator=g)
    print(f"[huge] nnz={nnz}", flush=True)
    plan = aes.aes_sample_build(rowptr, col, val, n_cols, W, 3, want_eid=True)
    Y = aes.aes_spmm_f32(plan, X)
    Yf = aes.aes_spmm_fused_f32(rowptr, col, val, n_cols, W, X, 3)
    torch.cuda.synchronize()
    assert torch.equal(Y, Yf)
    ref = orc.sample_build(rowptr.cpu().numpy(), col.cpu().numpy(), val.cpu().numpy(), W, seed=3)
    S = int(ref[0][-1])
    assert S == n_rows * W and int(ref[3].max()) > 2 ** 31
    assert np.array_equal(plan.s_rowptr.cpu().numpy(), ref[0])
    assert np.array_equal(plan.s_eid[:S].cpu().numpy(), ref[3])
    assert np.array_equal(plan.s_col[:S].cpu().numpy(), ref[1])
    assert np.array_equal(plan.s_val[:S].cpu().numpy().view(np.uint32), ref[2].view(np.uint32))
    G.check_f32(plan, ref, X)
