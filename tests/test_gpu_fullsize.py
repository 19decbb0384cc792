"""GPU parity at the benchmark's full sizes, in the launch configuration
bench.py times: the plan, the 8-bit codes and EVERY row of Y (float32 and 8-bit
features, every width of the configuration, the unsampled product where the
configuration names it) are compared with the oracle.  Only the fused layer and
the 111 M-node workload are compared on a seeded sample of rows."""
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


def _run(G, name, widths, exact=False, schemes=(SYM,), layer=False):
    from workloads import configs
    d = configs.make(name, "cuda")
    w = d["workload"]
    print(f"[{name}] n={d['n']} nnz={d['nnz']} F={d['F']}", flush=True)
    rowptr, col, val = (d[k].cpu().numpy() for k in ("rowptr", "colidx", "val"))
    X = d["X"]
    Xh = X.cpu().numpy()
    # row sample for the fused layer only (Y itself is compared on every row); it holds the longest rows too
    rows = np.sort(np.random.default_rng(1).choice(d["n"], size=min(N_ROWS_CHECKED, d["n"]), replace=False))
    rows = np.unique(np.concatenate([rows, np.argsort(np.diff(rowptr))[-8:]])).astype(np.int64)
    import paper_2503_18427_amd as aes
    q = {s: G.check_quantize(X, s, w.q_granularity) for s in schemes}
    deg = d["rowptr"][1:] - d["rowptr"][:-1]
    Y_exact = None
    for W in ((0,) if exact else ()) + tuple(widths):
        plan, ref = G.check_plan(d["rowptr"], d["colidx"], d["val"], d["n"], W, 0)
        Y, c, g = G.check_f32(plan, ref, X, rows=None, use_perm=False)        # all rows; bench.py's launch configuration
        print(f"[{name}] W={W} slots={int(ref[0][-1])} fp32 err on all {d['n']} rows comp={c:.2e} glob={g:.2e}", flush=True)
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
            _, c, g = G.check_q8(plan, ref, q[s][0], q[s][1], s, w.q_granularity, rows=None, use_perm=False)
            print(f"[{name}] W={W} int8 scheme={s} err on all rows comp={c:.2e} glob={g:.2e}", flush=True)
        if layer and W == widths[0]:
            _check_layer(G, name, d, plan, ref, Xh, q[SYM], w.q_granularity, rows)
        del plan, ref
    return d


def _check_layer(G, name, d, plan, ref, Xh, q, gran, rows, Fo=64):
    """The fused layer at full size: sampled rows of H against the oracle's aggregate-then-combine
    in double, for float32 features and for the symmetric 8-bit codes."""
    import oracle as orc
    import paper_2503_18427_amd as aes
    F = d["F"]
    Theta = (np.random.default_rng(3).standard_normal((F, Fo)) / np.sqrt(F)).astype(np.float32)
    Td = G.to_dev(Theta)
    rt = torch.from_numpy(rows).cuda()
    H = aes.aes_gcn_layer_f32(plan, d["X"], Td)
    Hq = aes.aes_gcn_layer_q8(plan, q[0][0], SYM, gran, q[0][1], q[0][2], Td)
    torch.cuda.synchronize()
    Yref, Yabs = orc.spmm_plan(ref[0], ref[1], ref[2], Xh, rows=rows, want_abs=True)
    Habs = orc.combine(Yabs, np.abs(Theta))
    e32 = float(np.max(np.abs(H[rt].cpu().numpy() - orc.combine(Yref, Theta)) / np.where(Habs > 0, Habs, 1.0)))
    Yqref, Yqabs = orc.spmm_q8(ref[0], ref[1], ref[2], q[1][0], SYM, gran, q[1][1], q[1][2], rows=rows, want_abs=True)
    Hqabs = orc.combine(Yqabs, np.abs(Theta))
    e8 = float(np.max(np.abs(Hq[rt].cpu().numpy() - orc.combine(Yqref, Theta)) / np.where(Hqabs > 0, Hqabs, 1.0)))
    print(f"[{name}] fused layer Fo={Fo}: fp32 err {e32:.2e}, int8 err {e8:.2e}", flush=True)
    assert e32 <= 2e-5 and e8 <= G.Q8_TOL      # 2e-5: two chained float32 sums (aggregation, MFMA product)


def test_arxiv_like(G):
    _run(G, "arxiv_like", (32, 64), schemes=(SYM, AFF), layer=True)


def test_products_like(G):
    _run(G, "products_like", (64,), schemes=(SYM,), layer=True)


def test_reddit_like(G):
    _run(G, "reddit_like", (64, 128, 256), exact=True, schemes=(SYM,), layer=True)


def test_rmat20(G):
    _run(G, "rmat20", (16, 32, 64, 128, 256), schemes=(SYM,))


def test_reddit_like_with_602_features(G):
    """The reddit-shaped graph at the width of the paper's Reddit features (602, Table 2): neither a
    multiple of 256 nor of 4, so the multiplies take their several-vectors-per-lane variants and the
    layer its general kernel, here over 233 000 rows instead of a few hundred.  Every row of Y
    (float32 and 8-bit), sampled rows of the fused layer."""
    from workloads import configs, graphs
    import paper_2503_18427_amd as aes
    w = configs.WORKLOADS["reddit_like"]
    rowptr, colidx, val = configs.make_graph(w, "cuda")
    F, W = 602, 64
    X = graphs.features(w.n, F, w.x_dist, w.seed + 1000, torch.device("cuda"))
    d = {"n": w.n, "F": F, "X": X}
    print(f"[reddit_like F=602] n={w.n} nnz={int(colidx.numel())}", flush=True)
    plan, ref = G.check_plan(rowptr, colidx, val, w.n, W, 0)
    Y, c, g = G.check_f32(plan, ref, X, use_perm=False)
    print(f"[reddit_like F=602] fp32 err on all rows comp={c:.2e} glob={g:.2e}", flush=True)
    assert torch.equal(aes.aes_spmm_fused_f32(rowptr, colidx, val, w.n, W, X), Y)
    q = G.check_quantize(X, SYM, w.q_granularity)
    _, c, g = G.check_q8(plan, ref, q[0], q[1], SYM, w.q_granularity, use_perm=False)
    print(f"[reddit_like F=602] int8 err on all rows comp={c:.2e} glob={g:.2e}", flush=True)
    rows = np.sort(np.random.default_rng(2).choice(w.n, size=N_ROWS_CHECKED, replace=False)).astype(np.int64)
    _check_layer(G, "reddit_like F=602", d, plan, ref, X.cpu().numpy(), q, w.q_granularity, rows, Fo=128)


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


def test_papers_like_scale(G):
    """111 M nodes, 1.66 G entries, 53 GB of float32 features on one GPU: every
    index path beyond 2^31 (entries, slots, feature elements).  The oracle runs on
    the sub-matrix of a seeded row sample (its CSR segments and the feature rows
    they touch are copied to the host), which is Algorithm 1 row by row."""
    import oracle as orc
    import paper_2503_18427_amd as aes
    from workloads import configs
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < 230 * 2 ** 30:
        pytest.skip("needs about 200 GiB of free GPU memory")
    d = configs.make("papers_like", "cuda")
    w = d["workload"]
    n, F, W = d["n"], d["F"], w.widths[0]
    rowptr, colidx, val, X = d["rowptr"], d["colidx"], d["val"], d["X"]
    print(f"[papers_like] n={n} nnz={d['nnz']}", flush=True)
    assert d["nnz"] > 2 ** 30 and n * F > 2 ** 33
    plan = aes.aes_sample_build(rowptr, colidx, val, n, W, 0)
    Y = aes.aes_spmm_f32(plan, X)
    q = aes.aes_quantize_features(X, SYM, w.q_granularity)
    Yq = aes.aes_spmm_q8(plan, q[0], SYM, w.q_granularity, q[1], q[2])
    torch.cuda.synchronize()
    rng = np.random.default_rng(0)
    deg = rowptr[1:] - rowptr[:-1]
    rows = np.unique(np.concatenate([rng.choice(n, 3000, replace=False), [0, n - 1, int(torch.argmax(deg))]]))
    rt = torch.from_numpy(rows).cuda()
    b, e = rowptr[rt], rowptr[rt + 1]
    seg = torch.cat([torch.arange(int(bb), int(ee), device="cuda") for bb, ee in zip(b.tolist(), e.tolist())])
    sub_rowptr = np.concatenate([[0], np.cumsum((e - b).cpu().numpy())]).astype(np.int64)
    sub_col, sub_val = colidx[seg].cpu().numpy(), val[seg].cpu().numpy()
    cols = np.unique(sub_col)                       # the feature rows the sampled rows can touch
    remap = np.full(n, -1, dtype=np.int64)
    remap[cols] = np.arange(cols.size)
    sub_col = remap[sub_col].astype(np.int32)
    ct = torch.from_numpy(cols).cuda()
    # plan rows: slot counts and sampled columns, bit for bit
    ref = orc.sample_build(sub_rowptr, sub_col, sub_val, W, 0)
    got_counts = (plan.s_rowptr[rt + 1] - plan.s_rowptr[rt]).cpu().numpy()
    assert np.array_equal(got_counts, np.diff(ref[0]))
    pseg = torch.cat([torch.arange(int(bb), int(ee), device="cuda")
                      for bb, ee in zip(plan.s_rowptr[rt].tolist(), plan.s_rowptr[rt + 1].tolist())])
    assert np.array_equal(remap[plan.s_col[pseg].cpu().numpy()], ref[1])
    assert np.array_equal(plan.s_val[pseg].cpu().numpy().view(np.uint32), ref[2].view(np.uint32))
    # products
    from helpers import rel_err
    Yref, Yabs = orc.spmm_plan(ref[0], ref[1], ref[2], X[ct].cpu().numpy(), want_abs=True)
    comp, glob = rel_err(Y[rt].cpu().numpy(), Yref, Yabs)
    print(f"[papers_like] fp32 err comp={comp:.2e} glob={glob:.2e}", flush=True)
    assert comp <= G.F32_TOL and glob <= G.F32_TOL
    rq, rs = q[0][ct].cpu().numpy(), q[1][ct].cpu().numpy()
    oq, os_, oz = orc.quantize(X[ct].cpu().numpy(), SYM, w.q_granularity)
    assert np.array_equal(rq, oq) and np.array_equal(rs.view(np.uint32), os_.view(np.uint32))
    Yqref, Yqabs = orc.spmm_q8(ref[0], ref[1], ref[2], oq, SYM, w.q_granularity, os_, oz, want_abs=True)
    comp, glob = rel_err(Yq[rt].cpu().numpy(), Yqref, Yqabs)
    print(f"[papers_like] int8 err comp={comp:.2e} glob={glob:.2e}", flush=True)
    assert comp <= G.Q8_TOL and glob <= G.Q8_TOL


def test_stated_maxima_of_F_and_W(G):
    """The largest feature width the entry points accept (2^24 - 1: odd, so the element-wise tail
    launch runs too) on a four-row matrix, and the largest sampling width (AES_MAX_W = 2^20) on a
    row of three million entries, which Table 1 samples down to 2^20 slots shared by the workgroup."""
    import paper_2503_18427_amd as aes
    rng = np.random.default_rng(9)
    F = 2 ** 24 - 1
    rowptr = np.array([0, 3, 3, 4, 9], dtype=np.int64)
    col = np.array([2, 0, 1, 1, 0, 2, 2, 1, 0], dtype=np.int32)
    val = rng.standard_normal(9).astype(np.float32)
    X = rng.standard_normal((3, F)).astype(np.float32)
    print("[maxima] F = 2^24 - 1", flush=True)
    plan, ref = G.check_plan(rowptr, col, val, 3, 4, 0)
    G.check_f32(plan, ref, X)
    qd, qr = G.check_quantize(X, SYM, 2)
    G.check_q8(plan, ref, qd, qr, SYM, 2)
    del X, qd, qr, plan, ref
    W = aes.AES_MAX_W
    deg = np.array([3_000_000, 5, 0, W, W + 1], dtype=np.int64)
    n_cols, F = 50_000, 96
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    col = rng.integers(0, n_cols, size=int(rowptr[-1])).astype(np.int32)
    val = rng.standard_normal(int(rowptr[-1])).astype(np.float32)
    X = rng.standard_normal((n_cols, F)).astype(np.float32)
    print("[maxima] W = 2^20", flush=True)
    plan, ref = G.check_plan(rowptr, col, val, n_cols, W, 0)
    assert int(ref[0][1]) == W and int(ref[0][-1] - ref[0][-2]) == W       # both long rows sampled to W slots
    Y, _, _ = G.check_f32(plan, ref, X)
    Yf = aes.aes_spmm_fused_f32(G.to_dev(rowptr), G.to_dev(col), G.to_dev(val), n_cols, W, G.to_dev(X))
    torch.cuda.synchronize()
    assert torch.equal(Y, Yf)


def test_column_indices_up_to_2_31(G):
    """n_cols = 2^31 - 1, the largest the entry points accept: gathers from feature rows whose index
    has bit 30 set, up to the last one, float32 (17 GB table, only the referenced rows are
    initialised and read) and 8-bit with per-column constants.  The oracle sees the referenced rows
    as a compact table."""
    import oracle as orc
    import paper_2503_18427_amd as aes
    from helpers import rel_err
    n_cols, F = 2 ** 31 - 1, 2
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < 30 * 2 ** 30:
        pytest.skip("needs about 22 GiB of free GPU memory")
    rng = np.random.default_rng(12)
    cols = np.array([0, 12345, 2 ** 30 - 1, 2 ** 30, 2 ** 30 + 77, 3 * 2 ** 29, 2 ** 31 - 3, 2 ** 31 - 2], dtype=np.int64)
    deg = np.array([5, 0, 8, 3, 70], dtype=np.int64)
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    pick = rng.integers(0, cols.size, size=int(rowptr[-1]))
    pick[:cols.size] = np.arange(cols.size)                  # every special column occurs
    col = cols[pick].astype(np.int32)
    val = rng.standard_normal(col.size).astype(np.float32)
    Xc = rng.standard_normal((cols.size, F)).astype(np.float32)
    print("[2^31 columns] allocating", flush=True)
    X = torch.empty((n_cols, F), dtype=torch.float32, device="cuda")
    X[torch.from_numpy(cols).cuda()] = torch.from_numpy(Xc).cuda()
    W = 16
    plan = aes.aes_sample_build(G.to_dev(rowptr), G.to_dev(col), G.to_dev(val), n_cols, W, 0)
    ref = orc.sample_build(rowptr, pick.astype(np.int32), val, W, seed=0)      # same plan over the compact table
    S = int(ref[0][-1])
    assert np.array_equal(plan.s_rowptr.cpu().numpy(), ref[0])
    assert np.array_equal(plan.s_col[:S].cpu().numpy(), cols[ref[1]].astype(np.int32))
    Y = aes.aes_spmm_f32(plan, X)
    Yf = aes.aes_spmm_fused_f32(G.to_dev(rowptr), G.to_dev(col), G.to_dev(val), n_cols, W, X)
    torch.cuda.synchronize()
    Yref, Yabs = orc.spmm_plan(ref[0], ref[1], ref[2], Xc, want_abs=True)
    comp, glob = rel_err(Y.cpu().numpy(), Yref, Yabs)
    assert comp <= G.F32_TOL and glob <= G.F32_TOL and torch.equal(Y, Yf), (comp, glob)
    del X
    q, s, z = orc.quantize(Xc, SYM, 1)
    Xq = torch.empty((n_cols, F), dtype=torch.int8, device="cuda")
    Xq[torch.from_numpy(cols).cuda()] = torch.from_numpy(q).cuda()
    Yq = aes.aes_spmm_q8(plan, Xq, SYM, 1, G.to_dev(s), G.to_dev(z))
    torch.cuda.synchronize()
    Yqref, Yqabs = orc.spmm_q8(ref[0], ref[1], ref[2], q, SYM, 1, s, z, want_abs=True)
    comp, glob = rel_err(Yq.cpu().numpy(), Yqref, Yqabs)
    assert comp <= G.Q8_TOL and glob <= G.Q8_TOL, (comp, glob)


def test_largest_leading_dimensions(G):
    """Feature matrices whose rows are 2^32 - 1 elements apart (the largest leading dimension the
    gathers accept) and an output whose rows are more than 2^32 elements apart: only the F
    columns in use are ever touched, so the buffers are allocated and never filled."""
    import oracle as orc
    import paper_2503_18427_amd as aes
    from helpers import rel_err
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < 130 * 2 ** 30:
        pytest.skip("needs about 100 GiB of free GPU memory")
    rng = np.random.default_rng(13)
    n_cols, F, ld = 3, 8, 2 ** 32 - 1
    rowptr = np.array([0, 4, 4, 9], dtype=np.int64)
    col = rng.integers(0, n_cols, size=9).astype(np.int32)
    val = rng.standard_normal(9).astype(np.float32)
    Xh = rng.standard_normal((n_cols, F)).astype(np.float32)
    print("[largest ld] allocating", flush=True)
    buf = torch.empty(((n_cols - 1) * ld + F,), dtype=torch.float32, device="cuda")
    X = torch.as_strided(buf, (n_cols, F), (ld, 1))
    X.copy_(torch.from_numpy(Xh).cuda())
    ldy = 2 ** 32 + 5
    ybuf = torch.empty((2 * ldy + F,), dtype=torch.float32, device="cuda")
    Y = torch.as_strided(ybuf, (3, F), (ldy, 1))
    plan, ref = G.check_plan(rowptr, col, val, n_cols, 4, 0)
    aes.aes_spmm_f32(plan, X, Y)
    torch.cuda.synchronize()
    Yref, Yabs = orc.spmm_plan(ref[0], ref[1], ref[2], Xh, want_abs=True)
    comp, glob = rel_err(Y.cpu().numpy(), Yref, Yabs)
    assert comp <= G.F32_TOL and glob <= G.F32_TOL, (comp, glob)
    # quantise from, and multiply with, the strided operands
    qbuf = torch.empty(((n_cols - 1) * ld + F,), dtype=torch.int8, device="cuda")
    Xq = torch.as_strided(qbuf, (n_cols, F), (ld, 1))
    rq, rs, rz = orc.quantize(Xh, SYM, 2)
    got = aes.aes_quantize_features(X, SYM, 2, out=(Xq, torch.empty(n_cols, device="cuda"), torch.empty(n_cols, device="cuda")))
    torch.cuda.synchronize()
    assert np.array_equal(got[0].cpu().numpy(), rq) and np.array_equal(got[1].cpu().numpy().view(np.uint32), rs.view(np.uint32))
    aes.aes_spmm_q8(plan, Xq, SYM, 2, got[1], got[2], Y)
    torch.cuda.synchronize()
    Yqref, Yqabs = orc.spmm_q8(ref[0], ref[1], ref[2], rq, SYM, 2, rs, rz, want_abs=True)
    comp, glob = rel_err(Y.cpu().numpy(), Yqref, Yqabs)
    assert comp <= G.Q8_TOL and glob <= G.Q8_TOL, (comp, glob)
