"""Small host-side helpers shared by the tests (no method arithmetic)."""
import numpy as np


def random_csr(n_rows, n_cols, degrees, rng, sort_cols=True):
    """CSR with the given per-row nnz; columns distinct within a row."""
    degrees = np.asarray(degrees, dtype=np.int64)
    rowptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(degrees, out=rowptr[1:])
    colidx = np.empty(rowptr[-1], dtype=np.int32)
    for r in range(n_rows):
        d = int(degrees[r])
        if d <= n_cols:
            c = rng.choice(n_cols, size=d, replace=False)
        else:
            c = rng.integers(0, n_cols, size=d)
        if sort_cols:
            c = np.sort(c)
        colidx[rowptr[r]:rowptr[r + 1]] = c
    val = rng.standard_normal(rowptr[-1]).astype(np.float32)
    return rowptr, colidx, val


def rel_err(Y, Yref, Yabs):
    """Componentwise |Y - Yref| / sum|terms| (0/0 -> 0) and max|d| / max|Yref|."""
    d = np.abs(Y.astype(np.float64) - Yref)
    denom = np.where(Yabs > 0, Yabs, 1.0)
    comp = float(np.max(d / denom)) if d.size else 0.0
    glob = float(d.max() / max(np.abs(Yref).max(), 1e-300)) if d.size else 0.0
    return comp, glob
