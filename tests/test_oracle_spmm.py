"""Pins of the oracle's multiply stage (Algorithm 1, Sec. 3.2): brute-force
dense products, reduction to exact CSR SpMM, and agreement of the one-pass and
the materialised forms."""
import numpy as np
import pytest
import scipy.sparse as sp

from helpers import random_csr


def _case(seed, n=180, n_cols=260, F=24, maxdeg=200):
    rng = np.random.default_rng(seed)
    deg = rng.integers(0, maxdeg, size=n)
    deg[:4] = [0, 1, maxdeg, 2]
    rowptr, col, val = random_csr(n, n_cols, deg, rng)
    X = rng.standard_normal((n_cols, F)).astype(np.float32)
    return rowptr, col, val, X


def _dense_from_elements(rowptr, eids, s_rowptr, col, val, n_cols):
    """Dense sampled matrix built slot by slot from source-element ids."""
    n = rowptr.size - 1
    A = np.zeros((n, n_cols), dtype=np.float64)
    for r in range(n):
        for e in eids[s_rowptr[r]:s_rowptr[r + 1]]:
            A[r, col[e]] += float(val[e])
    return A


@pytest.mark.parametrize("W", [4, 16, 32, 48, 64])
@pytest.mark.parametrize("seed", [0, 99])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_brute_force_dense(oracle, W, seed, mode):
    rowptr, col, val, X = _case(W)
    s_rowptr, s_col, s_val, s_eid = oracle.sample_build(rowptr, col, val, W, seed=seed, mode=mode)
    A = _dense_from_elements(rowptr, s_eid, s_rowptr, col, val, X.shape[0])
    Yd = A @ X.astype(np.float64)
    Y1, Yabs = oracle.spmm_plan(s_rowptr, s_col, s_val, X, want_abs=True)
    Y2 = oracle.aes_spmm(rowptr, col, val, W, X, seed=seed, mode=mode)
    tol = 1e-12 * np.maximum(Yabs, 1.0)
    assert np.all(np.abs(Y1 - Yd) <= tol)
    assert np.all(np.abs(Y2 - Yd) <= tol)
    Aabs = _dense_from_elements(rowptr, s_eid, s_rowptr, col, np.abs(val), X.shape[0])
    assert np.all(np.abs(Yabs - Aabs @ np.abs(X.astype(np.float64))) <= tol)


def test_wide_W_equals_exact_spmm(oracle):
    rowptr, col, val, X = _case(3)
    A = sp.csr_matrix((val.astype(np.float64), col, rowptr), shape=(rowptr.size - 1, X.shape[0]))
    Yex = A @ X.astype(np.float64)
    for W in [256, 1024, 0]:            # >= max degree, and the no-sampling path
        Y = oracle.aes_spmm(rowptr, col, val, W, X)
        assert np.allclose(Y, Yex, rtol=0, atol=1e-12)
        s = oracle.sample_build(rowptr, col, val, W)
        assert np.allclose(oracle.spmm_plan(s[0], s[1], s[2], X), Yex, rtol=0, atol=1e-12)


def test_short_rows_exact_long_rows_not(oracle):
    rowptr, col, val, X = _case(4)
    W = 32
    A = sp.csr_matrix((val.astype(np.float64), col, rowptr), shape=(rowptr.size - 1, X.shape[0]))
    Yex = A @ X.astype(np.float64)
    Y = oracle.aes_spmm(rowptr, col, val, W, X)
    deg = np.diff(rowptr)
    short = deg <= W
    assert np.allclose(Y[short], Yex[short], rtol=0, atol=1e-12)
    assert np.all(Y[deg == 0] == 0)
    # sampled rows really drop elements: they differ from the exact product
    assert np.any(np.abs(Y[~short] - Yex[~short]) > 1e-3)


def test_row_subset(oracle):
    rowptr, col, val, X = _case(6)
    rows = np.array([5, 0, 179, 2, 2, 77], dtype=np.int64)
    Yall = oracle.aes_spmm(rowptr, col, val, 16, X)
    assert np.array_equal(oracle.aes_spmm(rowptr, col, val, 16, X, rows=rows), Yall[rows])
    s = oracle.sample_build(rowptr, col, val, 16)
    assert np.array_equal(oracle.spmm_plan(s[0], s[1], s[2], X, rows=rows), Yall[rows])


def test_strided_features(oracle):
    rowptr, col, val, X = _case(8)
    buf = np.zeros((X.shape[0], X.shape[1] + 8), dtype=np.float32)
    buf[:, :X.shape[1]] = X
    Y0 = oracle.aes_spmm(rowptr, col, val, 16, X)
    assert np.array_equal(oracle.aes_spmm(rowptr, col, val, 16, buf[:, :X.shape[1]]), Y0)


def test_duplicates_are_added_again(oracle):
    """W = 64, row_nnz = 1436: every sample starts at 0 (modulus 1429), so the
    row's result is 8 x (first eight elements) - nothing de-duplicates."""
    nnz = 1436
    rowptr = np.array([0, nnz], dtype=np.int64)
    col = np.arange(nnz, dtype=np.int32)
    val = np.ones(nnz, dtype=np.float32)
    X = np.arange(nnz, dtype=np.float32).reshape(nnz, 1) + 1
    Y = oracle.aes_spmm(rowptr, col, val, 64, X)
    assert Y[0, 0] == 8 * sum(range(1, 9))


def test_workload_generator_smoke(oracle):
    from workloads import configs
    d = configs.make("tiny")
    rowptr, col, val = (d[k].numpy() for k in ("rowptr", "colidx", "val"))
    X = d["X"].numpy()
    assert rowptr[-1] == col.size and np.all(np.diff(rowptr) >= 1)     # self-loops
    for r in range(0, d["n"], 97):
        seg = col[rowptr[r]:rowptr[r + 1]]
        assert np.all(np.diff(seg) > 0)                                # ascending, distinct
    Y = oracle.aes_spmm(rowptr, col, val, 32, X)
    A = sp.csr_matrix((val.astype(np.float64), col, rowptr), shape=(d["n"], d["n"]))
    short = np.diff(rowptr) <= 32
    assert np.allclose(Y[short], (A @ X.astype(np.float64))[short], atol=1e-12)


def test_combination_phase_is_a_matrix_product(oracle):
    rng = np.random.default_rng(31)
    Y = rng.standard_normal((37, 20))
    Theta = rng.standard_normal((20, 13)).astype(np.float32)
    H = oracle.combine(Y, Theta)
    assert np.allclose(H, Y @ Theta.astype(np.float64), rtol=0, atol=1e-12)
    # non-square, so a transposed operand cannot pass; identity weights return Y
    assert np.array_equal(oracle.combine(Y, np.eye(20, dtype=np.float32)), Y)
