"""GPU parity: the HIP path through the C-ABI against the CPU oracle, element
by element, on seeded inputs that span several tiles and ragged tails, plus the
method's edge cases."""
import numpy as np
import pytest
import torch

from helpers import random_csr

pytestmark = pytest.mark.gpu

AFF, SYM = 0, 1
TENSOR, COLUMN, ROW = 0, 1, 2


@pytest.fixture(scope="module")
def G():
    import gpu_common
    import paper_2503_18427_amd as aes
    assert torch.cuda.is_available(), "these tests need the GPU"
    aes.library()
    return gpu_common


def _workload(name):
    from workloads import configs
    d = configs.make(name, "cpu")
    return (d["rowptr"].numpy(), d["colidx"].numpy(), d["val"].numpy(), d["X"].numpy(), d["workload"])


def _ragged_case(seed, W, n=700, F=64):
    rng = np.random.default_rng(seed)
    deg = rng.integers(0, 3 * max(W, 1) + 3, size=n)
    special = [0, 0, 1, max(W, 1), max(W, 1) + 1, 2 * max(W, 1), 2 * max(W, 1) + 1, 36 * max(W, 1),
               36 * max(W, 1) + 1, 54 * max(W, 1), 54 * max(W, 1) + 1, 1436, 5000]
    deg[:len(special)] = special
    rng.shuffle(deg)
    n_cols = 900
    rowptr, col, val = random_csr(n, n_cols, deg, rng)
    X = rng.standard_normal((n_cols, F)).astype(np.float32)
    return rowptr, col, val, X, n_cols


@pytest.mark.parametrize("W", [1, 2, 4, 7, 16, 32, 48, 64, 100, 128, 256, 1024, 0])
@pytest.mark.parametrize("seed", [0, 0x9E3779B97F4A7C15])
def test_sample_build_bit_exact(G, W, seed):
    rowptr, col, val, X, n_cols = _ragged_case(W + 1, W)
    plan, ref = G.check_plan(rowptr, col, val, n_cols, W, seed)
    G.check_f32(plan, ref, X)
    G.check_f32(plan, ref, X, use_perm=False)


@pytest.mark.parametrize("strategy", [0, 1, 2])
@pytest.mark.parametrize("W", [1, 4, 16, 48, 64, 256, 0])
@pytest.mark.parametrize("seed", [0, 77])
def test_strategies_and_fused_kernels(G, strategy, W, seed):
    """The fixed AFS / SFS granularities, and the single-kernel (sample on the
    fly) form: same slots and the same summation order as build + multiply, so
    the outputs must be bit-identical to the plan path."""
    import paper_2503_18427_amd as aes
    rowptr, col, val, X, n_cols = _ragged_case(W + 100 * strategy, W, n=500, F=96)
    plan, ref = G.check_plan(rowptr, col, val, n_cols, W, seed, strategy)
    Y, _, _ = G.check_f32(plan, ref, X, use_perm=False)
    d = [G.to_dev(a) for a in (rowptr, col, val)]
    Xd = G.to_dev(X)
    Yf = aes.aes_spmm_fused_f32(d[0], d[1], d[2], n_cols, W, Xd, seed, strategy=strategy)
    torch.cuda.synchronize()
    assert torch.equal(Yf, Y)
    for scheme, gran in ((SYM, ROW), (AFF, COLUMN), (SYM, TENSOR)):
        qd, qr = G.check_quantize(X, scheme, gran)
        Yq, _, _ = G.check_q8(plan, ref, qd, qr, scheme, gran, use_perm=False)
        Yqf = aes.aes_spmm_fused_q8(d[0], d[1], d[2], n_cols, W, qd[0], scheme, gran, qd[1], qd[2], seed,
                                    strategy=strategy)
        torch.cuda.synchronize()
        assert torch.equal(Yqf, Yq)
    # and against the oracle's own one-pass form
    import oracle as orc
    Yo, Yabs = orc.aes_spmm(rowptr, col, val, W, X, seed=seed, want_abs=True, mode=strategy)
    from helpers import rel_err
    comp, glob = rel_err(Yf.cpu().numpy(), Yo, Yabs)
    assert comp <= G.F32_TOL and glob <= G.F32_TOL


@pytest.mark.parametrize("name", ["tiny", "arxiv_small", "reddit_small", "products_small", "rmat12"])
def test_small_workloads(G, name):
    rowptr, col, val, X, w = _workload(name)
    xq = {}
    for scheme in (SYM, AFF):
        xq[scheme] = G.check_quantize(X, scheme, w.q_granularity)
    for W in w.widths + (0,):
        plan, ref = G.check_plan(rowptr, col, val, w.n, W, 0)
        Y1, c1, g1 = G.check_f32(plan, ref, X)
        Y2, _, _ = G.check_f32(plan, ref, X, use_perm=False)
        assert torch.equal(Y1, Y2)                   # row order does not change any sum
        for scheme in (SYM, AFF):
            G.check_q8(plan, ref, xq[scheme][0], xq[scheme][1], scheme, w.q_granularity)


@pytest.mark.parametrize("F", [1, 3, 4, 8, 20, 32, 50, 64, 100, 128, 192, 256, 260, 320, 512, 602, 777, 1024, 1100, 2053])
def test_feature_widths_and_alignment(G, F):
    rowptr, col, val, _, n_cols = _ragged_case(F, 32, n=300)
    rng = np.random.default_rng(F)
    X = rng.standard_normal((n_cols, F)).astype(np.float32)
    plan, ref = G.check_plan(rowptr, col, val, n_cols, 32, 0)
    G.check_f32(plan, ref, X)
    # padded leading dimension, and a view whose rows start at odd element offsets
    import paper_2503_18427_amd as aes
    buf = torch.zeros((n_cols, F + 9), device="cuda")
    buf[:, 1:F + 1] = G.to_dev(X)
    Yb = torch.full((rowptr.size - 1, F + 5), 7.0, device="cuda")
    aes.aes_spmm_f32(plan, buf[:, 1:F + 1], Yb[:, 2:F + 2])
    Y = aes.aes_spmm_f32(plan, G.to_dev(X))
    torch.cuda.synchronize()
    assert torch.equal(Yb[:, 2:F + 2], Y)
    assert torch.all(Yb[:, :2] == 7.0) and torch.all(Yb[:, F + 2:] == 7.0)   # padding untouched
    for scheme in (SYM, AFF):
        for gran in (TENSOR, COLUMN, ROW):
            qd, qr = G.check_quantize(X, scheme, gran)
            Yq, _, _ = G.check_q8(plan, ref, qd, qr, scheme, gran)
            # codes at an odd byte offset with an odd leading dimension: same bits
            qbuf = torch.zeros((n_cols, F + 3), dtype=qd[0].dtype, device="cuda")
            qbuf[:, 1:F + 1] = qd[0]
            Yb.fill_(7.0)
            aes.aes_spmm_q8(plan, qbuf[:, 1:F + 1], scheme, gran, qd[1], qd[2], Yb[:, 2:F + 2])
            torch.cuda.synchronize()
            assert torch.equal(Yb[:, 2:F + 2], Yq)
            assert torch.all(Yb[:, :2] == 7.0) and torch.all(Yb[:, F + 2:] == 7.0)


def test_quantize_layouts_and_constants(G):
    import paper_2503_18427_amd as aes
    rng = np.random.default_rng(9)
    n, F = 1000, 96
    X = (rng.standard_normal((n, F)) * 5).astype(np.float32)
    X[5, :] = 0.0                  # an all-zero row: scale 1 (symmetric), range 0 (affine)
    X[:, 7] = -2.5                 # a constant column
    X[17, 3] = 40.0
    for scheme in (SYM, AFF):
        for gran in (TENSOR, COLUMN, ROW):
            G.check_quantize(X, scheme, gran)
    # strided input and output
    big = torch.zeros((n, F + 12), device="cuda")
    big[:, 4:F + 4] = G.to_dev(X)
    outq = torch.zeros((n, F + 8), dtype=torch.int8, device="cuda")
    sc = torch.empty(n, device="cuda")
    zr = torch.empty(n, device="cuda")
    aes.aes_quantize_features(big[:, 4:F + 4], SYM, ROW, out=(outq[:, 4:F + 4], sc, zr))
    ref = aes.aes_quantize_features(G.to_dev(X), SYM, ROW)
    torch.cuda.synchronize()
    assert torch.equal(outq[:, 4:F + 4], ref[0]) and torch.equal(sc, ref[1])
    # rows at odd element / byte offsets with odd leading dimensions: same codes, padding untouched
    odd = torch.zeros((n, F + 7), device="cuda")
    odd[:, 3:F + 3] = G.to_dev(X)
    for scheme in (SYM, AFF):
        for gran in (TENSOR, COLUMN, ROW):
            want = aes.aes_quantize_features(G.to_dev(X), scheme, gran)
            oq = torch.full((n, F + 5), 77, dtype=want[0].dtype, device="cuda")
            groups = {TENSOR: 1, COLUMN: F, ROW: n}[gran]
            s2, z2 = torch.empty(groups, device="cuda"), torch.zeros(groups, device="cuda")
            aes.aes_quantize_features(odd[:, 3:F + 3], scheme, gran, out=(oq[:, 1:F + 1], s2, z2))
            back = torch.full((n, F + 7), 9.0, device="cuda")
            aes.aes_dequantize_features(oq[:, 1:F + 1], scheme, gran, s2, z2, back[:, 3:F + 3])
            torch.cuda.synchronize()
            assert torch.equal(oq[:, 1:F + 1], want[0]) and torch.equal(s2, want[1])
            assert torch.all(oq[:, :1] == 77) and torch.all(oq[:, F + 1:] == 77)
            assert torch.equal(back[:, 3:F + 3], aes.aes_dequantize_features(want[0], scheme, gran, want[1], want[2]))
            assert torch.all(back[:, :3] == 9.0) and torch.all(back[:, F + 3:] == 9.0)
    assert torch.all(outq[:, :4] == 0) and torch.all(outq[:, F + 4:] == 0)
    # constant tensor
    C = np.full((33, 8), 1.25, dtype=np.float32)
    G.check_quantize(C, AFF, TENSOR)
    G.check_quantize(np.zeros((33, 8), dtype=np.float32), SYM, COLUMN)


def test_empty_and_degenerate(G):
    import paper_2503_18427_amd as aes
    # no rows
    plan = aes.aes_sample_build(torch.zeros(1, dtype=torch.int64, device="cuda"),
                                torch.zeros(0, dtype=torch.int32, device="cuda"),
                                torch.zeros(0, device="cuda"), 5, 16)
    torch.cuda.synchronize()
    assert plan.s_rowptr.tolist() == [0]
    Y = aes.aes_spmm_f32(plan, torch.ones((5, 8), device="cuda"))
    assert Y.shape == (0, 8)
    # rows but no entries: zero output
    rowptr = np.zeros(1501, dtype=np.int64)
    plan, ref = G.check_plan(rowptr, np.zeros(0, np.int32), np.zeros(0, np.float32), 5, 16)
    Y = aes.aes_spmm_f32(plan, torch.ones((5, 8), device="cuda"), torch.full((1500, 8), 3.0, device="cuda"))
    torch.cuda.synchronize()
    assert torch.all(Y == 0)
    # one very long row and the all-starts-coincide row (modulus 1429)
    for nnz, W in [(100000, 64), (1436, 64), (1 << 17, 1024), (3_000_000, 65536), (2_000_000, 1 << 20)]:
        rp = np.array([0, nnz], dtype=np.int64)
        rng = np.random.default_rng(nnz)
        col = rng.integers(0, 300, size=nnz).astype(np.int32)
        val = rng.standard_normal(nnz).astype(np.float32)
        X = rng.standard_normal((300, 128)).astype(np.float32)
        plan, ref = G.check_plan(rp, col, val, 300, W)
        G.check_f32(plan, ref, X)
        plan0, ref0 = G.check_plan(rp, col, val, 300, 0)
        G.check_f32(plan0, ref0, X)


def test_bit_reproducible(G):
    import paper_2503_18427_amd as aes
    rowptr, col, val, X, w = _workload("products_small")
    plan, _ = G.check_plan(rowptr, col, val, w.n, 64)
    Xd = G.to_dev(X)
    Y1 = aes.aes_spmm_f32(plan, Xd).clone()
    Y2 = aes.aes_spmm_f32(plan, Xd)
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y2)


def test_side_stream(G):
    import paper_2503_18427_amd as aes
    rowptr, col, val, X, w = _workload("arxiv_small")
    plan, ref = G.check_plan(rowptr, col, val, w.n, 32)
    Xd = G.to_dev(X)
    Y0 = aes.aes_spmm_f32(plan, Xd)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        Y1 = aes.aes_spmm_f32(plan, Xd)
    s.synchronize()
    assert torch.equal(Y0, Y1)


def test_explicit_stream_argument_without_workspace(G):
    """`stream=` given explicitly (a torch stream, then its raw handle) and no workspace / output
    passed: everything the binding allocates must belong to that stream.  The allocations are
    provoked to be reused right away by work on the default stream; results must not change."""
    import paper_2503_18427_amd as aes
    rowptr, col, val, X, w = _workload("arxiv_small")
    d = [G.to_dev(a) for a in (rowptr, col, val)]
    Xd = G.to_dev(X)
    plan0 = aes.aes_sample_build(d[0], d[1], d[2], w.n, 32, 0)
    Y0 = aes.aes_spmm_f32(plan0, Xd)
    q0 = aes.aes_quantize_features(Xd, SYM, COLUMN)
    Yq0 = aes.aes_spmm_q8(plan0, q0[0], SYM, COLUMN, q0[1], q0[2])
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    for handle in (s, s.cuda_stream):
        s.wait_stream(torch.cuda.current_stream())
        plan = aes.aes_sample_build(d[0], d[1], d[2], w.n, 32, 0, stream=handle)
        Y = aes.aes_spmm_f32(plan, Xd, stream=handle)
        q = aes.aes_quantize_features(Xd, SYM, COLUMN, stream=handle)
        Yq = aes.aes_spmm_q8(plan, q[0], SYM, COLUMN, q[1], q[2], stream=handle)
        # default-stream work that would grab any block freed by the calls above
        junk = [torch.full((1 << 16,), float(i), device="cuda") for i in range(16)]
        s.synchronize()
        torch.cuda.synchronize()
        S = int(plan0.s_rowptr[-1].item())
        assert torch.equal(plan.s_rowptr, plan0.s_rowptr) and torch.equal(plan.s_col[:S], plan0.s_col[:S])
        assert torch.equal(Y, Y0) and torch.equal(q[0], q0[0]) and torch.equal(q[1], q0[1]) and torch.equal(Yq, Yq0)
        del junk


def test_hip_graph_capture_replays(G):
    """Every entry point only enqueues kernels on the caller's stream (no
    allocation, no memset, no synchronisation), so a whole step can be captured
    in a HIP graph; each replay must reproduce the eager results."""
    import paper_2503_18427_amd as aes
    rowptr, col, val, X, w = _workload("arxiv_small")
    d = [G.to_dev(a) for a in (rowptr, col, val)]
    Xd = G.to_dev(X)
    n, F, W = w.n, w.F, 32
    plan = aes.aes_sample_build(d[0], d[1], d[2], n, W, 0, want_perm=True)
    ws_b = torch.empty(aes.aes_sample_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    ws_q = torch.empty(max(aes.aes_quantize_workspace_bytes(n, F, COLUMN), 8), dtype=torch.uint8, device="cuda")
    qbuf = (torch.empty((n, F), dtype=torch.int8, device="cuda"), torch.empty(F, device="cuda"),
            torch.empty(F, device="cuda"))
    Y, Yq, Yf = (torch.empty((n, F), device="cuda") for _ in range(3))

    def step():
        aes.aes_sample_build(d[0], d[1], d[2], n, W, 0, out=plan, workspace=ws_b)
        aes.aes_spmm_f32(plan, Xd, Y)
        aes.aes_quantize_features(Xd, SYM, COLUMN, out=qbuf, workspace=ws_q)
        aes.aes_spmm_q8(plan, qbuf[0], SYM, COLUMN, qbuf[1], qbuf[2], Yq)
        aes.aes_spmm_fused_f32(d[0], d[1], d[2], n, W, Xd, Y=Yf)

    step()
    torch.cuda.synchronize()
    eager = [t.clone() for t in (plan.s_rowptr, plan.s_col, plan.s_val, Y, qbuf[0], Yq, Yf)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for t in (plan.s_col, plan.s_val, Y, Yq, Yf):
            t.fill_(-1)                          # eager work between replays
        qbuf[0].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        now = (plan.s_rowptr, plan.s_col, plan.s_val, Y, qbuf[0], Yq, Yf)
        S = int(plan.s_rowptr[-1])
        for a, b in zip(eager, now):
            if a.numel() == plan.s_col.numel() and a.dim() == 1:
                assert torch.equal(a[:S], b[:S]), rep
            else:
                assert torch.equal(a, b), rep


@pytest.mark.parametrize("F", [32, 96, 256, 320, 50, 602, 1300])
@pytest.mark.parametrize("W", [0, 4096])
def test_long_rows_shared_by_the_workgroup(G, F, W):
    """Rows above 2048 slots are split over all lane groups of a workgroup and
    summed in a fixed order: several such rows per workgroup, mixed with short
    and empty rows, every feature-chunk count, plan and fused forms, fp32 and
    8-bit, and bit-identical from run to run."""
    import paper_2503_18427_amd as aes
    rng = np.random.default_rng(F + W)
    deg = np.array([5000, 3, 2500, 0, 9000, 2049, 2048, 1, 70000, 64, 2047, 4097, 0, 33, 12000, 7] * 3)
    n, n_cols = deg.size, 1500
    rowptr, col, val = random_csr(n, n_cols, deg, rng)
    X = rng.standard_normal((n_cols, F)).astype(np.float32)
    plan, ref = G.check_plan(rowptr, col, val, n_cols, W, 0)
    Y, _, _ = G.check_f32(plan, ref, X, use_perm=False)
    Y2, _, _ = G.check_f32(plan, ref, X, use_perm=True)
    assert torch.equal(Y, Y2)
    d = [G.to_dev(a) for a in (rowptr, col, val)]
    Yf = aes.aes_spmm_fused_f32(d[0], d[1], d[2], n_cols, W, G.to_dev(X))
    Yr = aes.aes_spmm_f32(plan, G.to_dev(X), use_perm=False)
    torch.cuda.synchronize()
    assert torch.equal(Yf, Y) and torch.equal(Yr, Y)
    for scheme, gran in ((SYM, ROW), (AFF, ROW), (AFF, COLUMN), (SYM, COLUMN)):
        qd, qr = G.check_quantize(X, scheme, gran)
        Yq, _, _ = G.check_q8(plan, ref, qd, qr, scheme, gran, use_perm=False)
        Yqf = aes.aes_spmm_fused_q8(d[0], d[1], d[2], n_cols, W, qd[0], scheme, gran, qd[1], qd[2])
        torch.cuda.synchronize()
        assert torch.equal(Yqf, Yq)


@pytest.mark.parametrize("W", [0, 4096, 64])
@pytest.mark.parametrize("F", [128, 24])
def test_slot_counts_around_tile_and_unroll_boundaries(G, W, F):
    """Rows whose slot counts sit on and next to every internal boundary of the multiply: the 8-slot
    unrolled round, the 64-slot LDS tile, the 2048-slot hand-over to the whole workgroup; plan build,
    plan multiply, single-kernel form, fused layer."""
    import oracle as orc
    import paper_2503_18427_amd as aes
    rng = np.random.default_rng(W + F)
    deg = np.array([1, 7, 8, 9, 15, 16, 17, 55, 56, 57, 63, 64, 65, 71, 72, 73, 127, 128, 129, 191, 192, 193, 2040,
                    2047, 2048, 2049, 2055, 2056, 2057, 2111, 2112, 2113, 4095, 4096, 4097, 0])
    n, n_cols = deg.size, 1200
    rowptr, col, val = random_csr(n, n_cols, deg, rng)
    X = rng.standard_normal((n_cols, F)).astype(np.float32)
    plan, ref = G.check_plan(rowptr, col, val, n_cols, W, 0)
    Y, _, _ = G.check_f32(plan, ref, X, use_perm=False)
    d = [G.to_dev(a) for a in (rowptr, col, val)]
    Yf = aes.aes_spmm_fused_f32(d[0], d[1], d[2], n_cols, W, G.to_dev(X))
    torch.cuda.synchronize()
    assert torch.equal(Yf, Y)
    qd, qr = G.check_quantize(X, SYM, COLUMN)
    G.check_q8(plan, ref, qd, qr, SYM, COLUMN, use_perm=False)
    Theta = (rng.standard_normal((F, 40)) / np.sqrt(F)).astype(np.float32)
    H = aes.aes_gcn_layer_f32(plan, G.to_dev(X), G.to_dev(Theta))
    torch.cuda.synchronize()
    Yref, Yabs = orc.spmm_plan(ref[0], ref[1], ref[2], X, want_abs=True)
    Habs = orc.combine(Yabs, np.abs(Theta))
    err = np.abs(H.cpu().numpy() - orc.combine(Yref, Theta)) / np.where(Habs > 0, Habs, 1.0)
    assert float(err.max()) <= LAYER_TOL, float(err.max())


@pytest.mark.parametrize("F,Fo", [(128, 128), (256, 256), (64, 32), (32, 200), (100, 48), (8, 1), (256, 64), (128, 33)])
def test_gcn_layer_fused_with_matrix_cores(G, F, Fo):
    """Aggregation + combination in one kernel against the oracle (double), with
    rows that do not fill the last 32-row tile and output widths that do not fill
    the last 32-column MFMA block."""
    import oracle as orc
    import paper_2503_18427_amd as aes
    rowptr, col, val, _, n_cols = _ragged_case(F + Fo, 64, n=333)
    rng = np.random.default_rng(F * 1000 + Fo)
    X = rng.standard_normal((n_cols, F)).astype(np.float32)
    Theta = (rng.standard_normal((F, Fo)) / np.sqrt(F)).astype(np.float32)
    for W in (64, 0):
        plan, ref = G.check_plan(rowptr, col, val, n_cols, W, 0)
        H = aes.aes_gcn_layer_f32(plan, G.to_dev(X), G.to_dev(Theta))
        torch.cuda.synchronize()
        Y, Yabs = orc.spmm_plan(ref[0], ref[1], ref[2], X, want_abs=True)
        Href = orc.combine(Y, Theta)
        Habs = orc.combine(Yabs, np.abs(Theta))
        d = np.abs(H.cpu().numpy().astype(np.float64) - Href)
        comp = float(np.max(d / np.where(Habs > 0, Habs, 1.0)))
        assert comp <= LAYER_TOL, comp
        # strided operands and output
        Hb = torch.full((rowptr.size - 1, Fo + 3), 5.0, device="cuda")
        Tb = torch.zeros((F, Fo + 7), device="cuda")
        Tb[:, 2:Fo + 2] = G.to_dev(Theta)
        Xb = torch.zeros((n_cols, F + 5), device="cuda")
        Xb[:, 3:F + 3] = G.to_dev(X)
        aes.aes_gcn_layer_f32(plan, Xb[:, 3:F + 3], Tb[:, 2:Fo + 2], Hb[:, 1:Fo + 1])
        torch.cuda.synchronize()
        assert torch.equal(Hb[:, 1:Fo + 1], H)
        assert torch.all(Hb[:, 0] == 5.0) and torch.all(Hb[:, Fo + 1:] == 5.0)


LAYER_TOL = 2e-5    # fused layer, float32: two chained float32 sums (aggregation, then the MFMA product)


def _layer_reference(orc, ref, Xh, Theta):
    Y, Yabs = orc.spmm_plan(ref[0], ref[1], ref[2], Xh, want_abs=True)
    return orc.combine(Y, Theta), orc.combine(Yabs, np.abs(Theta))


@pytest.mark.parametrize("F,Fo", [(300, 40), (512, 128), (602, 200), (1024, 64), (6, 8), (260, 600), (30, 33), (129, 513)])
def test_gcn_layer_any_feature_width(G, F, Fo):
    """Feature widths beyond 256 and not multiples of four (the general kernel: features in chunks
    of 256 through LDS, MFMA accumulators kept across chunks), float32 and 8-bit, strided operands."""
    import oracle as orc
    import paper_2503_18427_amd as aes
    rowptr, col, val, _, n_cols = _ragged_case(F * 7 + Fo, 64, n=150)
    rng = np.random.default_rng(F * 1000 + Fo)
    X = (rng.standard_normal((n_cols, F)) * rng.uniform(0.2, 5.0, size=(n_cols, 1))).astype(np.float32)
    Theta = (rng.standard_normal((F, Fo)) / np.sqrt(F)).astype(np.float32)
    plan, ref = G.check_plan(rowptr, col, val, n_cols, 64, 0)
    Xb = torch.zeros((n_cols, F + 3), device="cuda")
    Xb[:, 1:F + 1] = G.to_dev(X)
    Tb = torch.zeros((F, Fo + 5), device="cuda")
    Tb[:, 2:Fo + 2] = G.to_dev(Theta)
    Hb = torch.full((rowptr.size - 1, Fo + 2), 5.0, device="cuda")
    aes.aes_gcn_layer_f32(plan, Xb[:, 1:F + 1], Tb[:, 2:Fo + 2], Hb[:, 1:Fo + 1])
    torch.cuda.synchronize()
    Href, Habs = _layer_reference(orc, ref, X, Theta)
    comp = float(np.max(np.abs(Hb[:, 1:Fo + 1].cpu().numpy() - Href) / np.where(Habs > 0, Habs, 1.0)))
    assert comp <= LAYER_TOL, comp
    assert torch.all(Hb[:, 0] == 5.0) and torch.all(Hb[:, Fo + 1:] == 5.0)
    for scheme, gran in ((SYM, COLUMN), (AFF, ROW), (AFF, COLUMN), (SYM, TENSOR)):
        qd, qr = G.check_quantize(X, scheme, gran)
        Hq = aes.aes_gcn_layer_q8(plan, qd[0], scheme, gran, qd[1], qd[2], G.to_dev(Theta))
        torch.cuda.synchronize()
        Y, Yabs = orc.spmm_q8(ref[0], ref[1], ref[2], qr[0], scheme, gran, qr[1], qr[2], want_abs=True)
        if scheme == AFF:
            sc = {0: qr[1][0], 1: qr[1][None, :], 2: qr[1][:, None]}[gran]
            zr = {0: qr[2][0], 1: qr[2][None, :], 2: qr[2][:, None]}[gran]
            mag = (np.abs(qr[0].astype(np.float32) * sc) + np.abs(zr)).astype(np.float32)
            Yabs = orc.spmm_plan(ref[0], ref[1], np.abs(ref[2]), np.ascontiguousarray(np.broadcast_to(mag, X.shape)))
        comp = float(np.max(np.abs(Hq.cpu().numpy() - orc.combine(Y, Theta)) /
                            np.where(orc.combine(Yabs, np.abs(Theta)) > 0, orc.combine(Yabs, np.abs(Theta)), 1.0)))
        assert comp <= G.Q8_TOL, (scheme, gran, comp)


@pytest.mark.parametrize("F", [128, 602])
def test_gcn_layer_long_rows(G, F):
    """Unsampled plan (W = 0) with a 70 000-slot row, rows just around the long-row threshold and
    empty rows: the long rows are shared by the workgroup with float64 partial sums."""
    import oracle as orc
    import paper_2503_18427_amd as aes
    rng = np.random.default_rng(F)
    deg = np.array([3, 70_000, 0, 2048, 2049, 17, 5000, 1] + [int(x) for x in rng.integers(0, 90, size=60)])
    n_cols = 3000
    rowptr, col, val = random_csr(deg.size, n_cols, deg, rng)
    X = rng.standard_normal((n_cols, F)).astype(np.float32)
    Theta = (rng.standard_normal((F, 48)) / np.sqrt(F)).astype(np.float32)
    plan, ref = G.check_plan(rowptr, col, val, n_cols, 0, 0)
    H = aes.aes_gcn_layer_f32(plan, G.to_dev(X), G.to_dev(Theta))
    torch.cuda.synchronize()
    Href, Habs = _layer_reference(orc, ref, X, Theta)
    comp = float(np.max(np.abs(H.cpu().numpy() - Href) / np.where(Habs > 0, Habs, 1.0)))
    assert comp <= LAYER_TOL, comp
    qd, qr = G.check_quantize(X, SYM, ROW)
    Hq = aes.aes_gcn_layer_q8(plan, qd[0], SYM, ROW, qd[1], qd[2], G.to_dev(Theta))
    torch.cuda.synchronize()
    Y, Yabs = orc.spmm_q8(ref[0], ref[1], ref[2], qr[0], SYM, ROW, qr[1], qr[2], want_abs=True)
    Hqabs = orc.combine(Yabs, np.abs(Theta))
    comp = float(np.max(np.abs(Hq.cpu().numpy() - orc.combine(Y, Theta)) / np.where(Hqabs > 0, Hqabs, 1.0)))
    assert comp <= G.Q8_TOL, comp
    # the layer is run-to-run reproducible (fixed summation order, no atomics)
    H2 = aes.aes_gcn_layer_f32(plan, G.to_dev(X), G.to_dev(Theta))
    torch.cuda.synchronize()
    assert torch.equal(H, H2)


def test_unsorted_rows_and_special_values(G):
    """Within-row order is the caller's (the sampler takes runs as stored), and
    non-finite features propagate exactly where the oracle says: only to rows
    that actually sample the poisoned feature row."""
    import oracle as orc
    import paper_2503_18427_amd as aes
    rng = np.random.default_rng(77)
    deg = rng.integers(0, 300, size=400)
    rowptr, col, val = random_csr(400, 700, deg, rng, sort_cols=False)
    X = rng.standard_normal((700, 64)).astype(np.float32)
    for W in (16, 64):
        plan, ref = G.check_plan(rowptr, col, val, 700, W, 0)
        G.check_f32(plan, ref, X, use_perm=False)
    Xp = X.copy()
    Xp[13, :] = np.nan
    Xp[500, 7] = np.inf
    Xp[600, 9] = -np.inf
    plan, ref = G.check_plan(rowptr, col, val, 700, 16, 0)
    Y = aes.aes_spmm_f32(plan, G.to_dev(Xp), use_perm=False).cpu().numpy()
    with np.errstate(invalid="ignore"):
        Yref = orc.spmm_plan(ref[0], ref[1], ref[2], Xp)
    assert np.array_equal(np.isnan(Y), np.isnan(Yref))
    assert np.array_equal(np.isposinf(Y), np.isposinf(Yref)) and np.array_equal(np.isneginf(Y), np.isneginf(Yref))
    ok = np.isfinite(Yref)
    assert np.isnan(Yref).any() and ok.any()
    assert np.max(np.abs(Y[ok] - Yref[ok])) < 1e-4


def test_two_streams_run_different_entry_points_concurrently(G):
    """No global state: calls on two streams with disjoint buffers may overlap."""
    import paper_2503_18427_amd as aes
    rowptr, col, val, X, w = _workload("products_small")
    d = [G.to_dev(a) for a in (rowptr, col, val)]
    Xd = G.to_dev(X)
    plan_a = aes.aes_sample_build(d[0], d[1], d[2], w.n, 64)
    Ya = aes.aes_spmm_f32(plan_a, Xd).clone()
    qa = aes.aes_quantize_features(Xd, SYM, ROW)
    Yqa = aes.aes_spmm_q8(plan_a, qa[0], SYM, ROW, qa[1], qa[2]).clone()
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for rep in range(4):
        with torch.cuda.stream(s1):
            p1 = aes.aes_sample_build(d[0], d[1], d[2], w.n, 64)
            y1 = aes.aes_spmm_f32(p1, Xd)
        with torch.cuda.stream(s2):
            q2 = aes.aes_quantize_features(Xd, SYM, ROW)
            y2 = aes.aes_spmm_q8(plan_a, q2[0], SYM, ROW, q2[1], q2[2])
        outs.append((p1, y1, q2, y2))
    s1.synchronize()
    s2.synchronize()
    for p1, y1, q2, y2 in outs:
        assert torch.equal(y1, Ya) and torch.equal(y2, Yqa) and torch.equal(q2[0], qa[0])


@pytest.mark.parametrize("scheme", [SYM, AFF])
@pytest.mark.parametrize("F", [128, 50])
def test_folded_row_constants(G, scheme, F):
    """Per-node dequantisation constants folded into the plan's values once: the
    8-bit product must still match the oracle's dequantise-then-multiply (and the
    unfolded kernel closely), on short, long and empty rows."""
    import paper_2503_18427_amd as aes
    rng = np.random.default_rng(F + scheme)
    deg = np.concatenate([rng.integers(0, 200, size=500), [0, 5000, 2049, 1, 64]])
    n_cols = 800
    rowptr, col, val = random_csr(deg.size, n_cols, deg, rng)
    X = (rng.standard_normal((n_cols, F)) * rng.uniform(0.1, 10.0, size=(n_cols, 1))).astype(np.float32)
    qd, qr = G.check_quantize(X, scheme, ROW)
    for W in (64, 0):
        plan, ref = G.check_plan(rowptr, col, val, n_cols, W, 0)
        Y0, _, _ = G.check_q8(plan, ref, qd, qr, scheme, ROW, use_perm=False)
        folded, bias = aes.aes_plan_fold_row_constants(plan, scheme, qd[1], qd[2])
        assert (bias is None) == (scheme == SYM)
        Yf = aes.aes_spmm_q8(folded, qd[0], scheme, aes.AES_Q_PER_ROW_FOLDED, None, bias, use_perm=False)
        torch.cuda.synchronize()
        # same check as the unfolded path: against the oracle's own dequantised product
        import oracle as orc
        from helpers import rel_err
        Yref, Yabs = orc.spmm_q8(ref[0], ref[1], ref[2], qr[0], scheme, ROW, qr[1], qr[2], want_abs=True)
        if scheme == AFF:
            mag = (np.abs(qr[0].astype(np.float32) * qr[1][:, None]) + np.abs(qr[2][:, None])).astype(np.float32)
            Yabs = orc.spmm_plan(ref[0], ref[1], np.abs(ref[2]), np.ascontiguousarray(mag))
        comp, glob = rel_err(Yf.cpu().numpy(), Yref, Yabs)
        assert comp <= G.Q8_TOL and glob <= G.Q8_TOL, (comp, glob)
        assert float((Yf - Y0).abs().max()) <= 1e-3 * max(1.0, float(Y0.abs().max()))
        # in place: the folded values may overwrite the plan's own
        S = int(plan.s_rowptr[-1])
        keep = plan.s_val.clone()
        aes.aes_plan_fold_row_constants(plan, scheme, qd[1], qd[2], s_val_folded=plan.s_val, row_bias=bias)
        torch.cuda.synchronize()
        assert torch.equal(plan.s_val[:S], folded.s_val[:S])
        plan.s_val.copy_(keep)


@pytest.mark.parametrize("scheme,gran", [(SYM, ROW), (SYM, COLUMN), (AFF, ROW), (AFF, COLUMN), (AFF, TENSOR), (SYM, TENSOR)])
@pytest.mark.parametrize("F,Fo", [(128, 64), (64, 100)])
def test_gcn_layer_on_8bit_features(G, scheme, gran, F, Fo):
    """The fused layer with the dequantisation inside the gather: against the oracle's
    dequantise -> aggregate -> combine in double, and with folded per-node constants."""
    import oracle as orc
    import paper_2503_18427_amd as aes
    rowptr, col, val, _, n_cols = _ragged_case(F + Fo + scheme + gran, 32, n=200)
    rng = np.random.default_rng(F + 7 * gran)
    X = (rng.standard_normal((n_cols, F)) * rng.uniform(0.2, 5.0, size=(n_cols, 1))).astype(np.float32)
    Theta = (rng.standard_normal((F, Fo)) / np.sqrt(F)).astype(np.float32)
    qd, qr = G.check_quantize(X, scheme, gran)
    plan, ref = G.check_plan(rowptr, col, val, n_cols, 32, 0)
    H = aes.aes_gcn_layer_q8(plan, qd[0], scheme, gran, qd[1], qd[2], G.to_dev(Theta))
    torch.cuda.synchronize()
    Y, Yabs = orc.spmm_q8(ref[0], ref[1], ref[2], qr[0], scheme, gran, qr[1], qr[2], want_abs=True)
    if scheme == AFF:
        sc = {0: qr[1][0], 1: qr[1][None, :], 2: qr[1][:, None]}[gran]
        zr = {0: qr[2][0], 1: qr[2][None, :], 2: qr[2][:, None]}[gran]
        mag = (np.abs(qr[0].astype(np.float32) * sc) + np.abs(zr)).astype(np.float32)
        Yabs = orc.spmm_plan(ref[0], ref[1], np.abs(ref[2]), np.ascontiguousarray(np.broadcast_to(mag, X.shape)))
    Href = orc.combine(Y, Theta)
    Habs = orc.combine(Yabs, np.abs(Theta))
    comp = float(np.max(np.abs(H.cpu().numpy() - Href) / np.where(Habs > 0, Habs, 1.0)))
    assert comp <= G.Q8_TOL, comp
    # the fused layer equals the 8-bit SpMM followed by a float64 product with Theta, closely
    Yg = aes.aes_spmm_q8(plan, qd[0], scheme, gran, qd[1], qd[2], use_perm=False)
    assert float((H.double() - Yg.double() @ G.to_dev(Theta).double()).abs().max()) < 1e-4
    if gran == ROW:
        fplan, bias = aes.aes_plan_fold_row_constants(plan, scheme, qd[1], qd[2])
        Hf = aes.aes_gcn_layer_q8(fplan, qd[0], scheme, aes.AES_Q_PER_ROW_FOLDED, None, bias, G.to_dev(Theta))
        torch.cuda.synchronize()
        assert float((Hf - H).abs().max()) < 1e-4


def test_random_shapes_sweep(G):
    """Two hundred seeded random combinations of graph shape (degree mixes with empty rows, rows
    around the tile, unroll and long-row boundaries, hubs), feature width, leading-dimension
    padding, W, seed, granularity and 8-bit scheme: plan bit-exact, both multiplies against the
    oracle, the one-kernel forms bit-identical to build + multiply, and every third case through
    the fused layer.  Sizes keep every output away from total cancellation (>= 17 rows, >= 64
    columns), so the whole-matrix error figure stays meaningful."""
    import oracle as orc
    import paper_2503_18427_amd as aes

    def degrees(rng, n):
        kind = int(rng.integers(0, 5))
        if kind == 0:
            return rng.integers(0, 12, size=n)
        if kind == 1:
            return rng.integers(0, 300, size=n)
        if kind == 2:
            return np.minimum((rng.pareto(1.2, size=n) * 4).astype(np.int64), 6000)
        if kind == 3:
            return rng.choice([0, 1, 2, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513, 1023, 1025, 2047,
                               2048, 2049], size=n)
        d = rng.integers(0, 40, size=n)
        d[rng.integers(0, n, size=max(1, n // 50))] = rng.integers(2000, 9000)
        return d

    widths = [1, 2, 3, 4, 5, 7, 8, 12, 16, 31, 32, 33, 60, 64, 100, 127, 128, 129, 192, 255, 256, 257, 300, 384, 511,
              512, 513, 602, 640, 768, 769, 1000, 1024, 1025, 1500]
    Ws = [0, 1, 2, 3, 4, 5, 8, 15, 16, 17, 31, 32, 33, 48, 64, 65, 100, 128, 200, 256, 512, 1000, 1024, 2048, 2049,
          3000, 4096]
    for case in range(200):
        rng = np.random.default_rng(20250318 + case)
        n = int(rng.choice([17, 63, 64, 65, 100, 255, 256, 257, 300]))
        n_cols = int(rng.choice([64, 333, 1000, 4000]))
        d = degrees(rng, n).astype(np.int64)
        if d.sum() > 300_000:
            d //= 4
        F, W = int(rng.choice(widths)), int(rng.choice(Ws))
        seed = int(rng.choice([0, 1, 2, 77, 0x9E3779B97F4A7C15, 2 ** 63 + 5]))
        strategy = int(rng.choice([0, 0, 0, 1, 2]))
        padl, padr = int(rng.integers(0, 4)), int(rng.integers(0, 6))
        scheme, gran = int(rng.choice([SYM, AFF])), int(rng.integers(0, 3))
        what = (case, n, n_cols, int(d.sum()), F, W, seed, strategy, padl, padr, scheme, gran)
        rowptr, col, val = random_csr(n, n_cols, d, rng, sort_cols=bool(rng.integers(0, 2)))
        X = (rng.standard_normal((n_cols, F)) * rng.uniform(0.1, 8.0, size=(n_cols, 1))).astype(np.float32)
        if rng.integers(0, 4) == 0:
            X[rng.integers(0, n_cols)] = 0.0
        try:
            plan, ref = G.check_plan(rowptr, col, val, n_cols, W, seed, strategy)
            Xb = torch.zeros((n_cols, F + padl + padr), device="cuda")
            Xb[:, padl:padl + F] = G.to_dev(X)
            Xv = Xb[:, padl:padl + F]
            use_perm = bool(rng.integers(0, 2))
            Y, _, _ = G.check_f32(plan, ref, Xv, use_perm=use_perm)
            csr = (G.to_dev(rowptr), G.to_dev(col), G.to_dev(val))
            Yf = aes.aes_spmm_fused_f32(*csr, n_cols, W, Xv, seed, strategy=strategy)
            assert torch.equal(Y, Yf), "one-kernel float32 form differs from build + multiply"
            qd, qr = G.check_quantize(X, scheme, gran)
            Yq, _, _ = G.check_q8(plan, ref, qd, qr, scheme, gran, use_perm=use_perm)
            Yqf = aes.aes_spmm_fused_q8(*csr, n_cols, W, qd[0], scheme, gran, qd[1], qd[2], seed, strategy=strategy)
            assert torch.equal(Yq, Yqf), "one-kernel 8-bit form differs from build + multiply"
            if case % 3 == 0:
                Fo = int(rng.choice([1, 7, 32, 33, 64, 100, 128, 256, 300, 513, 600]))
                Theta = (rng.standard_normal((F, Fo)) / np.sqrt(F)).astype(np.float32)
                H = aes.aes_gcn_layer_f32(plan, Xv, G.to_dev(Theta))
                torch.cuda.synchronize()
                Href, Habs = _layer_reference(orc, ref, X, Theta)
                comp = float(np.max(np.abs(H.cpu().numpy() - Href) / np.where(Habs > 0, Habs, 1.0)))
                assert comp <= LAYER_TOL, ("layer float32", Fo, comp)
                Hq = aes.aes_gcn_layer_q8(plan, qd[0], scheme, gran, qd[1], qd[2], G.to_dev(Theta))
                torch.cuda.synchronize()
                Yr, Ya = orc.spmm_q8(ref[0], ref[1], ref[2], qr[0], scheme, gran, qr[1], qr[2], want_abs=True)
                if scheme == AFF:
                    sc = {0: qr[1][0], 1: qr[1][None, :], 2: qr[1][:, None]}[gran]
                    zr = {0: qr[2][0], 1: qr[2][None, :], 2: qr[2][:, None]}[gran]
                    mag = np.zeros(X.shape, np.float32) + (np.abs(qr[0].astype(np.float32) * sc) + np.abs(zr))
                    Ya = orc.spmm_plan(ref[0], ref[1], np.abs(ref[2]), mag.astype(np.float32))
                Hqa = orc.combine(Ya, np.abs(Theta))
                comp = float(np.max(np.abs(Hq.cpu().numpy() - orc.combine(Yr, Theta)) / np.where(Hqa > 0, Hqa, 1.0)))
                assert comp <= G.Q8_TOL, ("layer 8-bit", Fo, comp)
        except AssertionError as e:
            raise AssertionError(f"case (index, n, n_cols, nnz, F, W, seed, strategy, pad, pad, scheme, gran) = {what}: {e}")


@pytest.mark.parametrize("scheme", [SYM, AFF])
@pytest.mark.parametrize("F", [100, 128, 30, 3, 602, 121, 500, 124, 1000, 1024, 1500, 8])
def test_constants_inside_the_rows(G, scheme, F):
    """AES_Q_PER_ROW_INLINE: a node's scale (and zero point) stored behind its codes in its own row.
    Codes and constants bit-exact against the oracle's per-node quantisation, the bytes of the row
    beyond them untouched; every consumer (both multiplies, the one-kernel form, the fused layer,
    the stand-alone Eq. 2 pass) gives bit for bit what it gives with the constants in arrays of
    their own, and so the oracle's result."""
    import oracle as orc
    import paper_2503_18427_amd as aes
    INLINE = aes.AES_Q_PER_ROW_INLINE
    rowptr, col, val, _, n_cols = _ragged_case(F + 31 * scheme, 16, n=300)
    rng = np.random.default_rng(F)
    X = (rng.standard_normal((n_cols, F)) * rng.uniform(0.2, 5.0, size=(n_cols, 1))).astype(np.float32)
    Xd = G.to_dev(X)
    ld = aes.aes_quantize_inline_ld(F, scheme)
    off = (F + 3) // 4 * 4
    assert ld % 128 == 0 and ld >= off + (8 if scheme == AFF else 4) and ld - 128 < off + (8 if scheme == AFF else 4)
    qdtype = torch.uint8 if scheme == AFF else torch.int8
    buf = torch.full((n_cols, ld), 0x5A, dtype=qdtype, device="cuda")
    Xq, scale, zero = aes.aes_quantize_features(Xd, scheme, INLINE, out=buf)
    torch.cuda.synchronize()
    rq, rs, rz = orc.quantize(X, scheme, ROW)
    assert np.array_equal(Xq.cpu().numpy(), rq), "codes"
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), rs.view(np.uint32)), "scale inside the rows"
    used = off + 4
    if scheme == AFF:
        assert np.array_equal(zero.cpu().numpy().view(np.uint32), rz.view(np.uint32)), "zero inside the rows"
        used += 4
    raw = buf.cpu().numpy().view(np.uint8)
    assert np.all(raw[:, F:off] == 0x5A) and np.all(raw[:, used:] == 0x5A), "bytes outside codes and constants were written"
    # the same constants in arrays of their own
    sep = aes.aes_quantize_features(Xd, scheme, ROW)
    assert torch.equal(sep[1], scale) and (scheme == SYM or torch.equal(sep[2], zero))
    plan, ref = G.check_plan(rowptr, col, val, n_cols, 16, 0)
    Y_in = aes.aes_spmm_q8(plan, Xq, scheme, INLINE, None)
    Y_sep, _, _ = G.check_q8(plan, ref, sep, (rq, rs, rz), scheme, ROW)
    # symmetric codes: the same operations in the same order wherever the scale comes from.  Affine: where the
    # lane group takes the constants from its own gather it adds the zero-point terms slot by slot instead of
    # lane by lane, so the two agree to rounding only; both are held to the oracle.
    if scheme == SYM:
        assert torch.equal(Y_in, Y_sep)
    else:
        Yref, _ = orc.spmm_q8(ref[0], ref[1], ref[2], rq, scheme, ROW, rs, rz, want_abs=True)
        mag = (np.abs(rq.astype(np.float32) * rs[:, None]) + np.abs(rz[:, None])).astype(np.float32)
        Yabs = orc.spmm_plan(ref[0], ref[1], np.abs(ref[2]), np.ascontiguousarray(mag))
        from helpers import rel_err
        comp, glob = rel_err(Y_in.cpu().numpy(), Yref, Yabs)
        assert comp <= G.Q8_TOL and glob <= G.Q8_TOL, (comp, glob)
        assert float((Y_in - Y_sep).abs().max()) <= 1e-5 * float(Y_sep.abs().max())
    csr = (G.to_dev(rowptr), G.to_dev(col), G.to_dev(val))
    assert torch.equal(aes.aes_spmm_fused_q8(*csr, n_cols, 16, Xq, scheme, INLINE, None), Y_in)
    Theta = G.to_dev((rng.standard_normal((F, 40)) / np.sqrt(F)).astype(np.float32))
    H_in = aes.aes_gcn_layer_q8(plan, Xq, scheme, INLINE, None, None, Theta)
    H_sep = aes.aes_gcn_layer_q8(plan, sep[0], scheme, ROW, sep[1], sep[2], Theta)
    if scheme == SYM:
        assert torch.equal(H_in, H_sep)
    else:
        assert float((H_in - H_sep).abs().max()) <= 2e-5 * float(H_sep.abs().max())
    Xhat = aes.aes_dequantize_features(Xq, scheme, INLINE, None)
    torch.cuda.synchronize()
    assert np.array_equal(Xhat.cpu().numpy().view(np.uint32), orc.dequantize(rq, scheme, ROW, rs, rz).view(np.uint32))
    # the unsampled plan: rows of 1436 and 5000 slots, the longer one shared by the workgroup (float64 partial sums)
    plan0, ref0 = G.check_plan(rowptr, col, val, n_cols, 0, 0)
    Y0_in = aes.aes_spmm_q8(plan0, Xq, scheme, INLINE, None)
    Y0_sep, _, _ = G.check_q8(plan0, ref0, sep, (rq, rs, rz), scheme, ROW)
    assert float((Y0_in - Y0_sep).abs().max()) <= 1e-5 * float(Y0_sep.abs().max())
    if scheme == SYM:
        assert torch.equal(Y0_in, Y0_sep)


def test_constants_inside_the_rows_single_node(G):
    """One feature row only (the row stride of a one-row matrix is not visible in its shape), and an empty matrix."""
    import paper_2503_18427_amd as aes
    INLINE = aes.AES_Q_PER_ROW_INLINE
    rng = np.random.default_rng(5)
    X = G.to_dev(rng.standard_normal((1, 100)).astype(np.float32))
    rowptr = np.array([0, 3, 3, 4], dtype=np.int64)
    col = np.zeros(4, dtype=np.int32)
    val = rng.standard_normal(4).astype(np.float32)
    plan = aes.aes_sample_build(G.to_dev(rowptr), G.to_dev(col), G.to_dev(val), 1, 8, 0)
    for scheme in (SYM, AFF):
        sep = aes.aes_quantize_features(X, scheme, ROW)
        inl = aes.aes_quantize_features(X, scheme, INLINE)
        assert torch.equal(inl[0], sep[0]) and torch.equal(inl[1], sep[1])
        Y_sep = aes.aes_spmm_q8(plan, sep[0], scheme, ROW, sep[1], sep[2])
        Y_in = aes.aes_spmm_q8(plan, inl[0], scheme, INLINE, None)
        assert float((Y_in - Y_sep).abs().max()) <= 1e-6 * float(Y_sep.abs().max())
        assert torch.equal(aes.aes_dequantize_features(inl[0], scheme, INLINE, None),
                           aes.aes_dequantize_features(sep[0], scheme, ROW, sep[1], sep[2]))
    empty = aes.aes_quantize_features(torch.empty((0, 100), device="cuda"), SYM, INLINE)
    assert empty[0].shape == (0, 100)
