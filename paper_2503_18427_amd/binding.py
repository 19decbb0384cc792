"""ctypes marshalling for libaes_spmm.so (see include/aes_spmm.h for semantics)."""
from __future__ import annotations

import ctypes
import functools
import os
from typing import NamedTuple, Optional

import torch

from . import build as _build

AES_OK, AES_ERR_INVALID_ARG, AES_ERR_UNSUPPORTED, AES_ERR_WORKSPACE, AES_ERR_HIP = 0, -1, -2, -3, -4
AES_Q_PER_TENSOR, AES_Q_PER_COLUMN, AES_Q_PER_ROW, AES_Q_PER_ROW_FOLDED, AES_Q_PER_ROW_INLINE = 0, 1, 2, 3, 4
AES_Q_AFFINE_FLOOR_U8, AES_Q_SYMMETRIC_RNE_I8 = 0, 1
AES_STRATEGY_ADAPTIVE, AES_STRATEGY_AFS, AES_STRATEGY_SFS = 0, 1, 2
AES_NOALLOC_MAX_ROWS = 1 << 24
AES_MAX_W = 1 << 20

_i64, _i32, _u64, _vp, _sz = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_size_t

# name -> (restype, argtypes); one entry per symbol declared in include/aes_spmm.h
SIGNATURES = {
    "aes_last_error": (ctypes.c_char_p, []),
    "aes_sample_capacity": (_i64, [_i64, _i64, _i32]),
    "aes_sample_workspace_bytes": (_sz, [_i64]),
    "aes_sample_build": (ctypes.c_int, [_i64, _i64, _i64, _vp, _vp, _vp, _i32, _u64, _i32, _vp, _vp, _vp, _vp, _vp,
                                        _vp, _sz, _vp]),
    "aes_sample_build_noalloc": (ctypes.c_int, [_i64, _i64, _i64, _vp, _vp, _vp, _i32, _u64, _i32, _vp, _vp, _vp, _vp,
                                                _vp, _vp]),
    "aes_spmm_fused_f32": (ctypes.c_int, [_i64, _i64, _vp, _vp, _vp, _i32, _u64, _i32, _vp, _i64, _i32, _vp, _i64,
                                          _vp]),
    "aes_spmm_fused_q8": (ctypes.c_int, [_i64, _i64, _vp, _vp, _vp, _i32, _u64, _i32, _vp, _i64, _i32, _i32, _i32,
                                         _vp, _vp, _vp, _i64, _vp]),
    "aes_spmm_f32": (ctypes.c_int, [_i64, _i64, _i32, _vp, _vp, _vp, _vp, _vp, _i64, _i32, _vp, _i64, _vp]),
    "aes_quantize_workspace_bytes": (_sz, [_i64, _i32, _i32]),
    "aes_quantize_inline_ld": (_i64, [_i32, _i32]),
    "aes_quantize_features": (ctypes.c_int, [_i64, _i32, _vp, _i64, _i32, _i32, _vp, _i64, _vp, _vp, _vp, _sz, _vp]),
    "aes_plan_fold_row_constants": (ctypes.c_int, [_i64, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp]),
    "aes_gcn_layer_f32": (ctypes.c_int, [_i64, _i64, _i32, _vp, _vp, _vp, _vp, _i64, _i32, _vp, _i64, _i32, _vp, _i64,
                                         _vp]),
    "aes_gcn_layer_q8": (ctypes.c_int, [_i64, _i64, _i32, _vp, _vp, _vp, _vp, _i64, _i32, _i32, _i32, _vp, _vp, _vp,
                                        _i64, _i32, _vp, _i64, _vp]),
    "aes_dequantize_features": (ctypes.c_int, [_i64, _i32, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _i64, _vp]),
    "aes_spmm_q8": (ctypes.c_int, [_i64, _i64, _i32, _vp, _vp, _vp, _vp, _vp, _i64, _i32, _i32, _i32, _vp, _vp, _vp,
                                   _i64, _vp]),
}

_lib = None


class AesError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"aes status {code}: {message}")
        self.code = code


def library() -> ctypes.CDLL:
    """The loaded shared library; built first if no build is present or if the build that is present
    was made from other sources than the ones beside it (a stale library is never loaded silently)."""
    global _lib
    if _lib is None:
        path = os.environ.get("AES_SPMM_LIBRARY")       # an explicitly named build is loaded as it is
        if not path:
            path = _build.lib_path()
            if not _build.is_current():
                _build.build()
        lib = ctypes.CDLL(path)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)          # AttributeError if a declared symbol is missing
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def aes_last_error() -> str:
    return library().aes_last_error().decode()


def _check(rc: int) -> None:
    if rc != AES_OK:
        raise AesError(rc, aes_last_error())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _on_stream(fn):
    """Runs a binding function with the caller's `stream=` as torch's current stream, so that every
    tensor the function allocates itself (outputs, workspaces) belongs to the stream its kernels
    run on: the caching allocator then cannot hand such a block to other work on another stream
    while those kernels still use it.  A raw hipStream_t handle (an int) is wrapped, not copied."""
    @functools.wraps(fn)
    def wrapper(*args, stream=None, **kwargs):
        if stream is None:
            return fn(*args, stream=None, **kwargs)
        s = stream if isinstance(stream, torch.cuda.Stream) else torch.cuda.ExternalStream(int(stream))
        with torch.cuda.stream(s):
            return fn(*args, stream=s, **kwargs)
    return wrapper


def _dev(t: torch.Tensor, dtype, name: str, dims: int = 1) -> torch.Tensor:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name}: a tensor in GPU memory is required")
    if t.dtype != dtype:
        raise TypeError(f"{name}: dtype {dtype} required, got {t.dtype}")
    if t.dim() != dims:
        raise TypeError(f"{name}: {dims}-d tensor required")
    if dims == 1 and t.numel() > 1 and t.stride(0) != 1:
        raise TypeError(f"{name}: must be contiguous")
    if dims == 2 and t.shape[1] > 1 and t.stride(1) != 1:
        raise TypeError(f"{name}: rows must be contiguous (unit stride along features)")
    return t


def _ld(t: torch.Tensor) -> int:
    return int(t.stride(0)) if t.shape[0] > 1 else max(int(t.shape[1]), 1)


def _ldq(Xq: torch.Tensor, granularity: int) -> int:
    """Leading dimension of a matrix of codes; with the constants inside the rows the view's own row stride
    counts even for a single row (the constants lie beyond the F columns of the view)."""
    if granularity == AES_Q_PER_ROW_INLINE:
        return max(int(Xq.stride(0)), int(Xq.shape[1]), 1)
    return _ld(Xq)


class Plan(NamedTuple):
    """The sampled matrix A_s as written by aes_sample_build (device tensors)."""
    n_rows: int
    n_cols: int
    W: int
    s_rowptr: torch.Tensor            # int64, n_rows + 1
    s_col: torch.Tensor               # int32, capacity; valid up to s_rowptr[-1]
    s_val: torch.Tensor               # float32, same
    s_eid: Optional[torch.Tensor]     # int64 or None
    row_perm: Optional[torch.Tensor]  # int32, n_rows, or None


def aes_sample_capacity(n_rows: int, nnz: int, W: int) -> int:
    cap = int(library().aes_sample_capacity(n_rows, nnz, W))
    if cap < 0:
        raise AesError(cap, aes_last_error())
    return cap


def aes_sample_workspace_bytes(n_rows: int) -> int:
    return int(library().aes_sample_workspace_bytes(n_rows))


def aes_quantize_workspace_bytes(n: int, F: int, granularity: int) -> int:
    return int(library().aes_quantize_workspace_bytes(n, F, granularity))


def aes_quantize_inline_ld(F: int, scheme: int) -> int:
    """Smallest multiple of 128 bytes that holds a row of F codes and its constants (AES_Q_PER_ROW_INLINE)."""
    ld = int(library().aes_quantize_inline_ld(int(F), int(scheme)))
    if ld < 0:
        raise AesError(ld, aes_last_error())
    return ld


def _inline_views(buf: torch.Tensor, F: int, scheme: int):
    """(Xq, scale, zero) as views of an n x ld byte buffer laid out for AES_Q_PER_ROW_INLINE."""
    off = (F + 3) // 4
    words = buf.view(torch.float32)
    return buf[:, :F], words[:, off], (words[:, off + 1] if scheme == AES_Q_AFFINE_FLOOR_U8 else None)


@_on_stream
def aes_sample_build(rowptr, colidx, val, n_cols: int, W: int, seed: int = 0, *,
                     strategy: int = AES_STRATEGY_ADAPTIVE, want_eid: bool = False,
                     want_perm: bool = False, out: Optional[Plan] = None, workspace=None, stream=None) -> Plan:
    """Build the sampled plan of a CSR matrix.  `out` reuses the buffers of an earlier plan.
    `want_perm` also asks for the class-ordered row permutation (a scheduling hint
    the SpMM calls use when `use_perm` is set; natural order measured faster on
    MI355X, so it is off by default)."""
    rowptr = _dev(rowptr, torch.int64, "rowptr")
    colidx = _dev(colidx, torch.int32, "colidx")
    val = _dev(val, torch.float32, "val")
    n_rows = rowptr.numel() - 1
    nnz = colidx.numel()
    if val.numel() != nnz:
        raise ValueError("colidx and val differ in length")
    dev = rowptr.device
    cap = aes_sample_capacity(n_rows, nnz, W)
    if out is None:
        out = Plan(n_rows, int(n_cols), int(W),
                   torch.empty(n_rows + 1, dtype=torch.int64, device=dev),
                   torch.empty(cap, dtype=torch.int32, device=dev),
                   torch.empty(cap, dtype=torch.float32, device=dev),
                   torch.empty(cap, dtype=torch.int64, device=dev) if want_eid else None,
                   torch.empty(n_rows, dtype=torch.int32, device=dev) if want_perm else None)
    elif out.s_rowptr.numel() != n_rows + 1 or out.s_col.numel() < cap or out.s_val.numel() < cap:
        raise ValueError("out: plan buffers too small")
    need = aes_sample_workspace_bytes(n_rows)
    if workspace is None:
        workspace = torch.empty(max(need, 8), dtype=torch.uint8, device=dev)
    _check(library().aes_sample_build(n_rows, int(n_cols), nnz, _ptr(rowptr), _ptr(colidx), _ptr(val), int(W),
                                      int(seed) & (2 ** 64 - 1), int(strategy), _ptr(out.s_rowptr), _ptr(out.s_col),
                                      _ptr(out.s_val), _ptr(out.s_eid), _ptr(out.row_perm), _ptr(workspace),
                                      workspace.numel(), _stream(stream)))
    return out._replace(n_rows=n_rows, n_cols=int(n_cols), W=int(W))


@_on_stream
def aes_sample_build_noalloc(rowptr, colidx, val, n_cols: int, W: int, seed: int = 0, *, out: Plan,
                             strategy: int = AES_STRATEGY_ADAPTIVE, stream=None) -> Plan:
    """aes_sample_build without a workspace and without any allocation: the plan buffers `out`
    are the caller's, the scratch is the library's built-in array (at most AES_NOALLOC_MAX_ROWS rows)."""
    rowptr, colidx, val = _csr(rowptr, colidx, val)
    n_rows = rowptr.numel() - 1
    nnz = colidx.numel()
    cap = aes_sample_capacity(n_rows, nnz, W)
    if out.s_rowptr.numel() < n_rows + 1 or out.s_col.numel() < cap or out.s_val.numel() < cap:
        raise ValueError("out: plan buffers too small")
    if (out.s_eid is not None and out.s_eid.numel() < cap) or (out.row_perm is not None and out.row_perm.numel() < n_rows):
        raise ValueError("out: s_eid / row_perm too small")
    _check(library().aes_sample_build_noalloc(n_rows, int(n_cols), nnz, _ptr(rowptr), _ptr(colidx), _ptr(val), int(W),
                                              int(seed) & (2 ** 64 - 1), int(strategy), _ptr(out.s_rowptr),
                                              _ptr(out.s_col), _ptr(out.s_val), _ptr(out.s_eid), _ptr(out.row_perm),
                                              _stream(stream)))
    return out._replace(n_rows=n_rows, n_cols=int(n_cols), W=int(W))


@_on_stream
def aes_spmm_f32(plan: Plan, X, Y=None, *, use_perm: bool = True, stream=None):
    """Y = A_s X for float32 features."""
    X = _dev(X, torch.float32, "X", 2)
    F = X.shape[1]
    if X.shape[0] != plan.n_cols:
        raise ValueError("X must have n_cols rows")
    if Y is None:
        Y = torch.empty((plan.n_rows, F), dtype=torch.float32, device=X.device)
    Y = _dev(Y, torch.float32, "Y", 2)
    if Y.shape[0] != plan.n_rows or Y.shape[1] != F:
        raise ValueError("Y has the wrong shape")
    perm = plan.row_perm if use_perm else None
    _check(library().aes_spmm_f32(plan.n_rows, plan.n_cols, plan.W, _ptr(plan.s_rowptr), _ptr(plan.s_col), _ptr(plan.s_val),
                                  _ptr(perm), _ptr(X), _ld(X), F, _ptr(Y), _ld(Y), _stream(stream)))
    return Y


@_on_stream
def aes_quantize_features(X, scheme: int, granularity: int, *, out=None, workspace=None, stream=None):
    """Returns (Xq, scale, zero); Xq is uint8 for the affine scheme, int8 for the symmetric one."""
    X = _dev(X, torch.float32, "X", 2)
    n, F = X.shape
    dev = X.device
    groups = {AES_Q_PER_TENSOR: 1, AES_Q_PER_COLUMN: F, AES_Q_PER_ROW: n}.get(granularity, 1)
    qdtype = torch.uint8 if scheme == AES_Q_AFFINE_FLOOR_U8 else torch.int8
    if granularity == AES_Q_PER_ROW_INLINE:
        # out: an n x ld byte buffer (ld from aes_quantize_inline_ld or larger); the results are views of it
        buf = out if out is not None else torch.empty((n, aes_quantize_inline_ld(F, scheme)), dtype=qdtype, device=dev)
        buf = _dev(buf, qdtype, "out", 2)
        if buf.shape[0] != n or not buf.is_contiguous() or buf.shape[1] % 4:
            raise ValueError("out: a contiguous n x ld buffer (ld a multiple of 4) is required for constants inside the rows")
        _check(library().aes_quantize_features(n, F, _ptr(X), _ld(X), int(scheme), int(granularity), _ptr(buf),
                                               buf.shape[1], None, None, None, 0, _stream(stream)))
        return _inline_views(buf, F, scheme)
    if out is None:
        out = (torch.empty((n, F), dtype=qdtype, device=dev),
               torch.empty(groups, dtype=torch.float32, device=dev),
               torch.empty(groups, dtype=torch.float32, device=dev))
    Xq, scale, zero = out
    need = aes_quantize_workspace_bytes(n, F, granularity)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    _check(library().aes_quantize_features(n, F, _ptr(X), _ld(X), int(scheme), int(granularity), _ptr(Xq), _ld(Xq),
                                           _ptr(scale), _ptr(zero), _ptr(workspace),
                                           0 if workspace is None else workspace.numel(), _stream(stream)))
    return Xq, scale, zero


@_on_stream
def aes_spmm_q8(plan: Plan, Xq, scheme: int, granularity: int, scale, zero=None, Y=None, *, use_perm: bool = True,
                stream=None):
    """Y = A_s x_hat with the dequantisation fused into the gather."""
    if not isinstance(Xq, torch.Tensor) or Xq.dtype not in (torch.int8, torch.uint8):
        raise TypeError("Xq: int8 / uint8 tensor required")
    Xq = _dev(Xq, Xq.dtype, "Xq", 2)
    if granularity == AES_Q_PER_ROW_INLINE:
        scale = zero = None                      # read from the rows of Xq
    if scale is not None:
        scale = _dev(scale, torch.float32, "scale")
    if zero is not None:
        zero = _dev(zero, torch.float32, "zero")
    F = Xq.shape[1]
    if Xq.shape[0] != plan.n_cols:
        raise ValueError("Xq must have n_cols rows")
    groups = {AES_Q_PER_TENSOR: 1, AES_Q_PER_COLUMN: F, AES_Q_PER_ROW: plan.n_cols}.get(granularity)
    if granularity == AES_Q_PER_ROW_FOLDED:
        if zero is not None and zero.numel() < plan.n_rows:
            raise ValueError("zero must hold the n_rows row biases for folded constants")
    elif groups is not None and (scale is None or scale.numel() < groups
                                 or (zero is not None and zero.numel() < groups)):
        raise ValueError("scale / zero too short for this granularity")
    if Y is None:
        Y = torch.empty((plan.n_rows, F), dtype=torch.float32, device=Xq.device)
    Y = _dev(Y, torch.float32, "Y", 2)
    if Y.shape[0] != plan.n_rows or Y.shape[1] != F:
        raise ValueError("Y has the wrong shape")
    perm = plan.row_perm if use_perm else None
    _check(library().aes_spmm_q8(plan.n_rows, plan.n_cols, plan.W, _ptr(plan.s_rowptr), _ptr(plan.s_col), _ptr(plan.s_val),
                                 _ptr(perm), _ptr(Xq), _ldq(Xq, granularity), F, int(scheme), int(granularity), _ptr(scale),
                                 _ptr(zero), _ptr(Y), _ld(Y), _stream(stream)))
    return Y


def _csr(rowptr, colidx, val):
    rowptr = _dev(rowptr, torch.int64, "rowptr")
    colidx = _dev(colidx, torch.int32, "colidx")
    val = _dev(val, torch.float32, "val")
    if val.numel() != colidx.numel():
        raise ValueError("colidx and val differ in length")
    return rowptr, colidx, val


@_on_stream
def aes_spmm_fused_f32(rowptr, colidx, val, n_cols: int, W: int, X, seed: int = 0, *,
                       strategy: int = AES_STRATEGY_ADAPTIVE, Y=None, stream=None):
    """Y = A_s X with the sampling done inside the SpMM kernel (no plan)."""
    rowptr, colidx, val = _csr(rowptr, colidx, val)
    X = _dev(X, torch.float32, "X", 2)
    n_rows, F = rowptr.numel() - 1, X.shape[1]
    if X.shape[0] != n_cols:
        raise ValueError("X must have n_cols rows")
    if Y is None:
        Y = torch.empty((n_rows, F), dtype=torch.float32, device=X.device)
    Y = _dev(Y, torch.float32, "Y", 2)
    if Y.shape[0] != n_rows or Y.shape[1] != F:
        raise ValueError("Y has the wrong shape")
    _check(library().aes_spmm_fused_f32(n_rows, int(n_cols), _ptr(rowptr), _ptr(colidx), _ptr(val), int(W),
                                        int(seed) & (2 ** 64 - 1), int(strategy), _ptr(X), _ld(X), F, _ptr(Y),
                                        _ld(Y), _stream(stream)))
    return Y


@_on_stream
def aes_spmm_fused_q8(rowptr, colidx, val, n_cols: int, W: int, Xq, scheme: int, granularity: int, scale,
                      zero=None, seed: int = 0, *, strategy: int = AES_STRATEGY_ADAPTIVE, Y=None, stream=None):
    """Fused sampling + 8-bit SpMM (no plan)."""
    rowptr, colidx, val = _csr(rowptr, colidx, val)
    if not isinstance(Xq, torch.Tensor) or Xq.dtype not in (torch.int8, torch.uint8):
        raise TypeError("Xq: int8 / uint8 tensor required")
    Xq = _dev(Xq, Xq.dtype, "Xq", 2)
    if granularity == AES_Q_PER_ROW_INLINE:
        scale = zero = None
    if scale is not None or granularity != AES_Q_PER_ROW_INLINE:
        scale = _dev(scale, torch.float32, "scale")
    if zero is not None:
        zero = _dev(zero, torch.float32, "zero")
    n_rows, F = rowptr.numel() - 1, Xq.shape[1]
    if Xq.shape[0] != n_cols:
        raise ValueError("Xq must have n_cols rows")
    groups = {AES_Q_PER_TENSOR: 1, AES_Q_PER_COLUMN: F, AES_Q_PER_ROW: int(n_cols)}.get(granularity)
    if groups is not None and (scale.numel() < groups or (zero is not None and zero.numel() < groups)):
        raise ValueError("scale / zero too short for this granularity")
    if Y is None:
        Y = torch.empty((n_rows, F), dtype=torch.float32, device=Xq.device)
    Y = _dev(Y, torch.float32, "Y", 2)
    if Y.shape[0] != n_rows or Y.shape[1] != F:
        raise ValueError("Y has the wrong shape")
    _check(library().aes_spmm_fused_q8(n_rows, int(n_cols), _ptr(rowptr), _ptr(colidx), _ptr(val), int(W),
                                       int(seed) & (2 ** 64 - 1), int(strategy), _ptr(Xq), _ldq(Xq, granularity), F, int(scheme),
                                       int(granularity), _ptr(scale), _ptr(zero), _ptr(Y), _ld(Y),
                                       _stream(stream)))
    return Y


@_on_stream
def aes_dequantize_features(Xq, scheme: int, granularity: int, scale, zero=None, X=None, *, stream=None):
    """Eq. 2 as a separate pass: float32 features from 8-bit codes."""
    if not isinstance(Xq, torch.Tensor) or Xq.dtype not in (torch.int8, torch.uint8):
        raise TypeError("Xq: int8 / uint8 tensor required")
    Xq = _dev(Xq, Xq.dtype, "Xq", 2)
    if granularity == AES_Q_PER_ROW_INLINE:
        scale = zero = None
    if scale is not None or granularity != AES_Q_PER_ROW_INLINE:
        scale = _dev(scale, torch.float32, "scale")
    if zero is not None:
        zero = _dev(zero, torch.float32, "zero")
    n, F = Xq.shape
    groups = {AES_Q_PER_TENSOR: 1, AES_Q_PER_COLUMN: F, AES_Q_PER_ROW: n}.get(granularity)
    if groups is not None and (scale.numel() < groups or (zero is not None and zero.numel() < groups)):
        raise ValueError("scale / zero too short for this granularity")
    if X is None:
        X = torch.empty((n, F), dtype=torch.float32, device=Xq.device)
    X = _dev(X, torch.float32, "X", 2)
    if X.shape != Xq.shape:
        raise ValueError("X has the wrong shape")
    _check(library().aes_dequantize_features(n, F, _ptr(Xq), _ldq(Xq, granularity), int(scheme), int(granularity), _ptr(scale),
                                             _ptr(zero), _ptr(X), _ld(X), _stream(stream)))
    return X


@_on_stream
def aes_gcn_layer_f32(plan: Plan, X, Theta, H=None, *, stream=None):
    """H = (A_s X) Theta in one kernel (aggregation + combination of a layer)."""
    X = _dev(X, torch.float32, "X", 2)
    Theta = _dev(Theta, torch.float32, "Theta", 2)
    F, Fo = X.shape[1], Theta.shape[1]
    if X.shape[0] != plan.n_cols or Theta.shape[0] != F:
        raise ValueError("X must be n_cols x F and Theta F x Fo")
    if H is None:
        H = torch.empty((plan.n_rows, Fo), dtype=torch.float32, device=X.device)
    H = _dev(H, torch.float32, "H", 2)
    if H.shape[0] != plan.n_rows or H.shape[1] != Fo:
        raise ValueError("H has the wrong shape")
    _check(library().aes_gcn_layer_f32(plan.n_rows, plan.n_cols, plan.W, _ptr(plan.s_rowptr), _ptr(plan.s_col),
                                       _ptr(plan.s_val), _ptr(X), _ld(X), F, _ptr(Theta), _ld(Theta), Fo, _ptr(H),
                                       _ld(H), _stream(stream)))
    return H


@_on_stream
def aes_plan_fold_row_constants(plan: Plan, scheme: int, scale, zero=None, *, s_val_folded=None, row_bias=None,
                                stream=None):
    """Fold per-node dequantisation constants into a plan.  Returns (folded plan, row_bias or None);
    use them with aes_spmm_q8(..., granularity=AES_Q_PER_ROW_FOLDED, scale=None, zero=row_bias)."""
    scale = _dev(scale, torch.float32, "scale")
    if zero is not None:
        zero = _dev(zero, torch.float32, "zero")
    if scale.numel() < plan.n_cols or (zero is not None and zero.numel() < plan.n_cols):
        raise ValueError("scale / zero must have one entry per column of the plan")
    if s_val_folded is None:
        s_val_folded = torch.empty_like(plan.s_val)
    affine = scheme == AES_Q_AFFINE_FLOOR_U8
    if affine and row_bias is None:
        row_bias = torch.empty(plan.n_rows, dtype=torch.float32, device=plan.s_val.device)
    _check(library().aes_plan_fold_row_constants(plan.n_rows, _ptr(plan.s_rowptr), _ptr(plan.s_col), _ptr(plan.s_val),
                                                 int(scheme), _ptr(scale), _ptr(zero), _ptr(s_val_folded),
                                                 _ptr(row_bias) if affine else None, _stream(stream)))
    return plan._replace(s_val=s_val_folded), (row_bias if affine else None)


@_on_stream
def aes_gcn_layer_q8(plan: Plan, Xq, scheme: int, granularity: int, scale, zero, Theta, H=None, *, stream=None):
    """H = (A_s x_hat) Theta with 8-bit features dequantised inside the gather."""
    if not isinstance(Xq, torch.Tensor) or Xq.dtype not in (torch.int8, torch.uint8):
        raise TypeError("Xq: int8 / uint8 tensor required")
    Xq = _dev(Xq, Xq.dtype, "Xq", 2)
    Theta = _dev(Theta, torch.float32, "Theta", 2)
    if granularity == AES_Q_PER_ROW_INLINE:
        scale = zero = None
    if scale is not None:
        scale = _dev(scale, torch.float32, "scale")
    if zero is not None:
        zero = _dev(zero, torch.float32, "zero")
    F, Fo = Xq.shape[1], Theta.shape[1]
    if Xq.shape[0] != plan.n_cols or Theta.shape[0] != F:
        raise ValueError("Xq must be n_cols x F and Theta F x Fo")
    groups = {AES_Q_PER_TENSOR: 1, AES_Q_PER_COLUMN: F, AES_Q_PER_ROW: plan.n_cols}.get(granularity)
    if groups is not None and (scale is None or scale.numel() < groups or (zero is not None and zero.numel() < groups)):
        raise ValueError("scale / zero too short for this granularity")
    if H is None:
        H = torch.empty((plan.n_rows, Fo), dtype=torch.float32, device=Xq.device)
    H = _dev(H, torch.float32, "H", 2)
    if H.shape[0] != plan.n_rows or H.shape[1] != Fo:
        raise ValueError("H has the wrong shape")
    _check(library().aes_gcn_layer_q8(plan.n_rows, plan.n_cols, plan.W, _ptr(plan.s_rowptr), _ptr(plan.s_col),
                                      _ptr(plan.s_val), _ptr(Xq), _ldq(Xq, granularity), F, int(scheme), int(granularity),
                                      _ptr(scale), _ptr(zero), _ptr(Theta), _ld(Theta), Fo, _ptr(H), _ld(H),
                                      _stream(stream)))
    return H
