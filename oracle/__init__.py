"""numpy front end of the CPU oracle (``aes_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
benchmark's cpu_baseline leg, never by the product package.  It holds no
arithmetic of its own; every function marshals numpy arrays into the C oracle.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "aes_oracle.c")
_LIB = os.path.join(_HERE, "libaes_oracle.so")

Q_PER_TENSOR, Q_PER_COLUMN, Q_PER_ROW = 0, 1, 2
Q_AFFINE_FLOOR_U8, Q_SYMMETRIC_RNE_I8 = 0, 1
STRATEGY_ADAPTIVE, STRATEGY_AFS, STRATEGY_SFS = 0, 1, 2

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  No fast-math, no FMA contraction."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, u64, i32, vp = ctypes.c_int64, ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p
        lib.orc_num_threads.restype = i32
        lib.orc_set_num_threads.argtypes = [i32]
        lib.orc_strategy.argtypes = [i64, i64, vp, vp]
        lib.orc_strategy_mode.argtypes = [i64, i64, i32, vp, vp]
        lib.orc_row_offset.argtypes = [u64, i64]
        lib.orc_row_offset.restype = ctypes.c_uint32
        lib.orc_hash.argtypes = [u64, i64, i64]
        lib.orc_hash.restype = i64
        lib.orc_row_slots.argtypes = [i64, i64, i32]
        lib.orc_row_slots.restype = i64
        lib.orc_sample_rowptr.argtypes = [i64, vp, i64, i32, vp]
        lib.orc_sample_build.argtypes = [i64, vp, vp, vp, i64, u64, i32, vp, vp, vp, vp]
        lib.orc_spmm_plan.argtypes = [i64, vp, vp, vp, vp, vp, i64, i64, vp, vp, i64]
        lib.orc_aes_spmm.argtypes = [i64, vp, vp, vp, vp, i64, u64, i32, vp, i64, i64, vp, vp, i64]
        lib.orc_aes_spmm.restype = i32
        lib.orc_combine.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64]
        lib.orc_quantize.argtypes = [i64, i64, vp, i64, i32, i32, vp, i64, vp, vp]
        lib.orc_quantize.restype = i32
        lib.orc_dequantize.argtypes = [i64, i64, vp, i64, i32, i32, vp, vp, vp, i64]
        lib.orc_dequantize.restype = i32
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def num_threads() -> int:
    return int(_load().orc_num_threads())


def set_num_threads(n: int) -> None:
    _load().orc_set_num_threads(int(n))


def strategy(row_nnz: int, W: int, mode: int = STRATEGY_ADAPTIVE):
    """(N, sample_cnt): Table 1 (mode 0) or the fixed AFS / SFS granularities."""
    n = ctypes.c_int64()
    c = ctypes.c_int64()
    if mode == STRATEGY_ADAPTIVE:
        _load().orc_strategy(int(row_nnz), int(W), ctypes.addressof(n), ctypes.addressof(c))
    else:
        _load().orc_strategy_mode(int(row_nnz), int(W), int(mode), ctypes.addressof(n), ctypes.addressof(c))
    return int(n.value), int(c.value)


def row_offset(seed: int, rid: int) -> int:
    return int(_load().orc_row_offset(int(seed), int(rid)))


def hash_start(current_ind: int, row_nnz: int, N: int) -> int:
    """start_ind of Eq. 3."""
    return int(_load().orc_hash(int(current_ind), int(row_nnz), int(N)))


def row_slots(row_nnz: int, W: int, mode: int = STRATEGY_ADAPTIVE) -> int:
    return int(_load().orc_row_slots(int(row_nnz), int(W), int(mode)))


def sample_build(rowptr, colidx, val, W: int, seed: int = 0, want_eid: bool = True,
                 mode: int = STRATEGY_ADAPTIVE):
    """Materialised sampled matrix.  Returns (s_rowptr, s_col, s_val, s_eid)."""
    lib = _load()
    rowptr = _c(rowptr, np.int64)
    colidx = _c(colidx, np.int32)
    val = _c(val, np.float32)
    n = rowptr.shape[0] - 1
    s_rowptr = np.empty(n + 1, dtype=np.int64)
    lib.orc_sample_rowptr(n, _p(rowptr), int(W), int(mode), _p(s_rowptr))
    S = int(s_rowptr[n])
    s_col = np.empty(S, dtype=np.int32)
    s_val = np.empty(S, dtype=np.float32)
    s_eid = np.empty(S, dtype=np.int64) if want_eid else None
    lib.orc_sample_build(n, _p(rowptr), _p(colidx), _p(val), int(W), int(seed), int(mode),
                         _p(s_rowptr), _p(s_col), _p(s_val), _p(s_eid))
    return s_rowptr, s_col, s_val, s_eid


def spmm_plan(s_rowptr, s_col, s_val, X, rows=None, want_abs: bool = False):
    """Y (float64) of the multiply stage on a plan; optionally also sum |terms|."""
    lib = _load()
    s_rowptr = _c(s_rowptr, np.int64)
    s_col = _c(s_col, np.int32)
    s_val = _c(s_val, np.float32)
    assert X.dtype == np.float32 and X.ndim == 2 and X.strides[1] == 4
    ldx = X.strides[0] // 4
    F = X.shape[1]
    if rows is not None:
        rows = _c(rows, np.int64)
        n = rows.shape[0]
    else:
        n = s_rowptr.shape[0] - 1
    Y = np.empty((n, F), dtype=np.float64)
    Yabs = np.empty((n, F), dtype=np.float64) if want_abs else None
    lib.orc_spmm_plan(n, _p(rows), _p(s_rowptr), _p(s_col), _p(s_val), _p(X), ldx, F,
                      _p(Y), _p(Yabs), F)
    return (Y, Yabs) if want_abs else Y


def aes_spmm(rowptr, colidx, val, W: int, X, seed: int = 0, rows=None, want_abs: bool = False,
             mode: int = STRATEGY_ADAPTIVE):
    """Algorithm 1 in one pass from the CSR.  W <= 0: exact SpMM."""
    lib = _load()
    rowptr = _c(rowptr, np.int64)
    colidx = _c(colidx, np.int32)
    val = _c(val, np.float32)
    assert X.dtype == np.float32 and X.ndim == 2 and X.strides[1] == 4
    ldx = X.strides[0] // 4
    F = X.shape[1]
    if rows is not None:
        rows = _c(rows, np.int64)
        n = rows.shape[0]
    else:
        n = rowptr.shape[0] - 1
    Y = np.empty((n, F), dtype=np.float64)
    Yabs = np.empty((n, F), dtype=np.float64) if want_abs else None
    rc = lib.orc_aes_spmm(n, _p(rows), _p(rowptr), _p(colidx), _p(val), int(W), int(seed), int(mode),
                          _p(X), ldx, F, _p(Y), _p(Yabs), F)
    if rc != 0:
        raise MemoryError("oracle scratch allocation failed")
    return (Y, Yabs) if want_abs else Y


def combine(Y, Theta):
    """H = Y @ Theta in double (the combination phase of a layer)."""
    lib = _load()
    Y = np.ascontiguousarray(Y, dtype=np.float64)
    Theta = np.ascontiguousarray(Theta, dtype=np.float32)
    n, F = Y.shape
    Fo = Theta.shape[1]
    assert Theta.shape[0] == F
    H = np.empty((n, Fo), dtype=np.float64)
    lib.orc_combine(n, F, Fo, _p(Y), F, _p(Theta), Fo, _p(H), Fo)
    return H


def _groups(n, F, granularity):
    return {Q_PER_TENSOR: 1, Q_PER_COLUMN: F, Q_PER_ROW: n}[granularity]


def quantize(X, scheme: int, granularity: int):
    """Returns (Xq, scale, zero).  Xq is int8 (symmetric) or uint8 (affine)."""
    lib = _load()
    assert X.dtype == np.float32 and X.ndim == 2 and X.strides[1] == 4
    n, F = X.shape
    ldx = X.strides[0] // 4 if n > 1 else max(F, 1)
    G = _groups(n, F, granularity)
    Xq = np.empty((n, F), dtype=np.int8)
    scale = np.empty(G, dtype=np.float32)
    zero = np.empty(G, dtype=np.float32)
    rc = lib.orc_quantize(n, F, _p(X), ldx, int(scheme), int(granularity), _p(Xq), F,
                          _p(scale), _p(zero))
    if rc != 0:
        raise ValueError("oracle quantize: bad arguments")
    if scheme == Q_AFFINE_FLOOR_U8:
        Xq = Xq.view(np.uint8)
    return Xq, scale, zero


def dequantize(Xq, scheme: int, granularity: int, scale, zero):
    """x_hat (float32) of Eq. 2."""
    lib = _load()
    assert Xq.dtype in (np.int8, np.uint8) and Xq.ndim == 2 and Xq.strides[1] == 1
    n, F = Xq.shape
    ldq = Xq.strides[0] if n > 1 else max(F, 1)
    scale = _c(scale, np.float32)
    zero = _c(zero if zero is not None else np.zeros_like(scale), np.float32)
    Xhat = np.empty((n, F), dtype=np.float32)
    rc = lib.orc_dequantize(n, F, _p(Xq), ldq, int(scheme), int(granularity), _p(scale),
                            _p(zero), _p(Xhat), F)
    if rc != 0:
        raise ValueError("oracle dequantize: bad arguments")
    return Xhat


def spmm_q8(s_rowptr, s_col, s_val, Xq, scheme, granularity, scale, zero, rows=None,
            want_abs: bool = False):
    """Quantised path: Eq. 2 in binary32, then the multiply stage in double."""
    Xhat = dequantize(Xq, scheme, granularity, scale, zero)
    return spmm_plan(s_rowptr, s_col, s_val, Xhat, rows=rows, want_abs=want_abs)
