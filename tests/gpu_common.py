"""Shared machinery of the GPU parity tests: run the HIP path through the
C-ABI binding and the CPU oracle on the same arrays and compare."""
import numpy as np
import torch

import oracle as orc
import paper_2503_18427_amd as aes
from helpers import rel_err

F32_TOL = 1e-5      # max relative error of Y, float32 features (target stated for this build)
Q8_TOL = 1e-2       # same for the 8-bit path, against the oracle's own dequantised product


def to_dev(a):
    if isinstance(a, torch.Tensor):
        return a.cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_host(a):
    return a.cpu().numpy() if isinstance(a, torch.Tensor) else a


def class_order(slots):
    """Rows by decreasing bit length of the slot count, original order within a class."""
    cls = np.zeros(slots.shape, dtype=np.int64)
    nz = slots > 0
    cls[nz] = np.floor(np.log2(slots[nz])).astype(np.int64) + 1
    return np.argsort(-cls, kind="stable").astype(np.int32)


def check_plan(rowptr, colidx, val, n_cols, W, seed=0, strategy=0):
    """aes_sample_build against the oracle, bit for bit.  Returns (plan, oracle plan)."""
    ref = orc.sample_build(to_host(rowptr), to_host(colidx), to_host(val), W, seed=seed, mode=strategy)
    plan = aes.aes_sample_build(to_dev(rowptr), to_dev(colidx), to_dev(val), n_cols, W, seed,
                                strategy=strategy, want_eid=True, want_perm=True)
    torch.cuda.synchronize()
    S = int(ref[0][-1])
    assert np.array_equal(plan.s_rowptr.cpu().numpy(), ref[0]), "s_rowptr"
    assert np.array_equal(plan.s_col[:S].cpu().numpy(), ref[1]), "s_col"
    assert np.array_equal(plan.s_val[:S].cpu().numpy().view(np.uint32), ref[2].view(np.uint32)), "s_val bits"
    assert np.array_equal(plan.s_eid[:S].cpu().numpy(), ref[3]), "s_eid"
    perm = plan.row_perm.cpu().numpy()
    assert np.array_equal(perm, class_order(np.diff(ref[0]))), "row_perm"
    return plan, ref


def check_f32(plan, ref, X, rows=None, use_perm=True, tol=F32_TOL):
    """aes_spmm_f32 against the oracle's multiply stage (double accumulation)."""
    Xd = X if isinstance(X, torch.Tensor) else to_dev(X)
    Xh = Xd.cpu().numpy() if isinstance(X, torch.Tensor) else X
    Y = aes.aes_spmm_f32(plan, Xd, use_perm=use_perm)
    torch.cuda.synchronize()
    Yh = Y.cpu().numpy()
    Yref, Yabs = orc.spmm_plan(ref[0], ref[1], ref[2], Xh, rows=rows, want_abs=True)
    got = Yh if rows is None else Yh[rows]
    comp, glob = rel_err(got, Yref, Yabs)
    assert comp <= tol and glob <= tol, (comp, glob)
    return Y, comp, glob


def check_quantize(X, scheme, gran):
    """aes_quantize_features against the oracle, bit for bit."""
    Xd = X if isinstance(X, torch.Tensor) else to_dev(X)
    Xh = Xd.cpu().numpy() if isinstance(X, torch.Tensor) else X
    Xq, scale, zero = aes.aes_quantize_features(Xd, scheme, gran)
    torch.cuda.synchronize()
    rq, rs, rz = orc.quantize(np.ascontiguousarray(Xh), scheme, gran)
    assert np.array_equal(Xq.cpu().numpy(), rq), "codes"
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), rs.view(np.uint32)), "scale"
    assert np.array_equal(zero.cpu().numpy(), rz), "zero"
    # Eq. 2 as a stand-alone pass: bit-identical to the oracle's dequantisation
    Xhat = aes.aes_dequantize_features(Xq, scheme, gran, scale, zero)
    torch.cuda.synchronize()
    ref_hat = orc.dequantize(rq, scheme, gran, rs, rz)
    assert np.array_equal(Xhat.cpu().numpy().view(np.uint32), ref_hat.view(np.uint32)), "x_hat"
    return (Xq, scale, zero), (rq, rs, rz)


def check_q8(plan, ref, q_dev, q_ref, scheme, gran, rows=None, use_perm=True, tol=Q8_TOL):
    """aes_spmm_q8 against dequantise-then-multiply done by the oracle."""
    Xq, scale, zero = q_dev
    Y = aes.aes_spmm_q8(plan, Xq, scheme, gran, scale, zero, use_perm=use_perm)
    torch.cuda.synchronize()
    Yh = Y.cpu().numpy()
    Yref, Yabs = orc.spmm_q8(ref[0], ref[1], ref[2], q_ref[0], scheme, gran, q_ref[1], q_ref[2], rows=rows,
                             want_abs=True)
    if scheme == orc.Q_AFFINE_FLOOR_U8:
        # x_hat = q*scale + zero is itself a difference of two rounded terms, so the
        # rounding error of a row scales with sum |v| (|q*scale| + |zero|), not with the
        # (possibly cancelling) |v * x_hat|: that is the denominator for this scheme.
        n, F = q_ref[0].shape
        sc = {0: q_ref[1][0], 1: q_ref[1][None, :], 2: q_ref[1][:, None]}[gran]
        zr = {0: q_ref[2][0], 1: q_ref[2][None, :], 2: q_ref[2][:, None]}[gran]
        mag = (np.abs(q_ref[0].astype(np.float32) * sc) + np.abs(zr)).astype(np.float32)
        Yabs = orc.spmm_plan(ref[0], ref[1], np.abs(ref[2]), np.ascontiguousarray(mag), rows=rows)
    got = Yh if rows is None else Yh[rows]
    comp, glob = rel_err(got, Yref, Yabs)
    assert comp <= tol and glob <= tol, (comp, glob)
    return Y, comp, glob
