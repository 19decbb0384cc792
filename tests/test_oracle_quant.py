"""Pins of the oracle's quantiser (Sec. 2.3, Eq. 1 and Eq. 2): closed forms,
error bounds, grouping, and binary32 evaluation order."""
import numpy as np
import pytest

AFF, SYM = 0, 1
TENSOR, COLUMN, ROW = 0, 1, 2


def test_affine_closed_form_unit_range(oracle):
    """x_min = 0, x_max = 1: q = floor(255 x).  For x = k/256 the product
    255k/256 is exact in binary32, so q = k - 1 for k >= 1 and q(0) = 0."""
    k = np.arange(256, dtype=np.float32)
    X = np.concatenate([k / 256.0, [1.0]]).astype(np.float32).reshape(1, -1)
    Xq, scale, zero = oracle.quantize(X, AFF, TENSOR)
    assert Xq.dtype == np.uint8
    exp = np.concatenate([[0], np.arange(1, 256) - 1, [255]])
    assert Xq[0].tolist() == exp.tolist()
    assert zero[0] == 0.0 and scale[0] == np.float32(1.0) / np.float32(255.0)


def test_affine_endpoints_and_bound(oracle):
    rng = np.random.default_rng(1)
    X = (rng.standard_normal((300, 40)) * 3 + 1).astype(np.float32)
    for gran in (TENSOR, COLUMN, ROW):
        Xq, scale, zero = oracle.quantize(X, AFF, gran)
        Xhat = oracle.dequantize(Xq, AFF, gran, scale, zero)
        if gran == TENSOR:
            lo, hi, sc = X.min(), X.max(), scale[0]
            assert Xq[X == lo].max() == 0 and Xq[X == hi].min() == 255
            assert zero[0] == lo
            err = X.astype(np.float64) - Xhat
        elif gran == COLUMN:
            assert np.array_equal(zero, X.min(axis=0))
            assert np.all(Xq[X.argmax(axis=0), np.arange(40)] == 255)
            assert np.all(Xq[X.argmin(axis=0), np.arange(40)] == 0)
            sc = scale[None, :]
            err = X.astype(np.float64) - Xhat
        else:
            assert np.array_equal(zero, X.min(axis=1))
            assert np.all(Xq[np.arange(300), X.argmax(axis=1)] == 255)
            sc = scale[:, None]
            err = X.astype(np.float64) - Xhat
        # Eq. 1 floors: reconstruction never overshoots by more than rounding,
        # and undershoots by less than one step
        slack = 4 * np.finfo(np.float32).eps * np.abs(X).max()
        assert np.all(err > -slack - 1e-3 * sc)
        assert np.all(err < sc * (1 + 1e-3) + slack)


def test_affine_constant_group(oracle):
    X = np.full((5, 3), 2.5, dtype=np.float32)
    Xq, scale, zero = oracle.quantize(X, AFF, TENSOR)
    assert np.all(Xq == 0) and scale[0] == 0 and zero[0] == 2.5
    assert np.all(oracle.dequantize(Xq, AFF, TENSOR, scale, zero) == 2.5)


def test_symmetric_ties_round_to_even(oracle):
    X = np.array([[127.0, -127.0, 0.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5, 125.5, 0.49, 3.51]],
                 dtype=np.float32)
    Xq, scale, zero = oracle.quantize(X, SYM, TENSOR)
    assert Xq.dtype == np.int8 and scale[0] == 1.0
    assert Xq[0].tolist() == [127, -127, 0, 0, 2, 2, 0, -2, -2, 126, 126, 0, 4]


def test_symmetric_bound_and_idempotence(oracle):
    rng = np.random.default_rng(2)
    X = rng.standard_normal((257, 33)).astype(np.float32)
    X[7, :] = 0
    for gran in (TENSOR, COLUMN, ROW):
        Xq, scale, zero = oracle.quantize(X, SYM, gran)
        Xhat = oracle.dequantize(Xq, SYM, gran, scale, zero)
        sc = {TENSOR: scale[0], COLUMN: scale[None, :], ROW: scale[:, None]}[gran]
        assert np.all(np.abs(X.astype(np.float64) - Xhat) <= 0.5 * sc * (1 + 1e-5))
        assert Xq.min() >= -127 and Xq.max() <= 127
        a = {TENSOR: np.abs(X).max(), COLUMN: np.abs(X).max(axis=0), ROW: np.abs(X).max(axis=1)}[gran]
        exp_scale = np.where(a == 0, np.float32(1), (a / np.float32(127)).astype(np.float32))
        assert np.array_equal(scale, np.atleast_1d(exp_scale).astype(np.float32))
        # quantising the reconstruction with the same scale returns the same codes
        t = (Xhat / sc).astype(np.float32)
        assert np.array_equal(np.clip(np.rint(t), -127, 127).astype(np.int8), Xq)
    Xq, scale, _ = oracle.quantize(X, SYM, ROW)
    assert scale[7] == 1.0 and np.all(Xq[7] == 0)


def test_grouping_orientation(oracle):
    """Column c holds values up to c+1, so per-column scales are (c+1)/127 and
    per-row scales are all F/127: a transposed grouping fails."""
    n, F = 6, 4
    X = np.zeros((n, F), dtype=np.float32)
    X[0, :] = np.arange(1, F + 1)
    X[1:, :] = 0.25
    _, sc_col, _ = oracle.quantize(X, SYM, COLUMN)
    assert sc_col.tolist() == [np.float32(c + 1) / np.float32(127) for c in range(F)]
    _, sc_row, _ = oracle.quantize(X, SYM, ROW)
    assert sc_row.tolist() == [np.float32(F) / np.float32(127)] + [np.float32(0.25) / np.float32(127)] * (n - 1)


def test_binary32_operation_order(oracle):
    """numpy float32 arithmetic performs the same IEEE operations one by one:
    divide, multiply, floor (affine); divide, round-half-even (symmetric);
    multiply, add (Eq. 2).  Catches double promotion and fused contraction."""
    rng = np.random.default_rng(3)
    X = (rng.standard_normal((500, 16)) * 10).astype(np.float32)
    Xq, scale, zero = oracle.quantize(X, AFF, COLUMN)
    lo, hi = X.min(axis=0), X.max(axis=0)
    d = (hi - lo).astype(np.float32)
    t = ((X - lo).astype(np.float32) / d).astype(np.float32) * np.float32(255)
    assert np.array_equal(Xq, np.clip(np.floor(t.astype(np.float32)), 0, 255).astype(np.uint8))
    assert np.array_equal(scale, (d / np.float32(255)).astype(np.float32))
    Xhat = oracle.dequantize(Xq, AFF, COLUMN, scale, zero)
    exp = (Xq.astype(np.float32) * scale).astype(np.float32) + zero
    assert np.array_equal(Xhat, exp.astype(np.float32))
    Xq2, scale2, _ = oracle.quantize(X, SYM, ROW)
    t2 = (X / scale2[:, None]).astype(np.float32)
    assert np.array_equal(Xq2, np.clip(np.rint(t2), -127, 127).astype(np.int8))


def test_q8_spmm_is_dequantise_then_multiply(oracle):
    rng = np.random.default_rng(4)
    n, F = 50, 12
    X = rng.standard_normal((n, F)).astype(np.float32)
    rowptr = np.arange(0, 3 * n + 1, 3, dtype=np.int64)
    col = rng.integers(0, n, size=3 * n).astype(np.int32)
    val = rng.standard_normal(3 * n).astype(np.float32)
    Xq, scale, zero = oracle.quantize(X, SYM, ROW)
    Y = oracle.spmm_q8(rowptr, col, val, Xq, SYM, ROW, scale, zero)
    A = np.zeros((n, n))
    np.add.at(A, (np.repeat(np.arange(n), 3), col), val.astype(np.float64))
    Xhat = Xq.astype(np.float64) * scale[:, None].astype(np.float64)
    assert np.allclose(Y, A @ Xhat, rtol=0, atol=1e-6)
    # and the quantised product is close to the fp32-feature product
    Yf = A @ X.astype(np.float64)
    assert np.max(np.abs(Y - Yf)) < 0.05
