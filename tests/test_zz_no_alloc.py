"""aes_sample_build_noalloc (the entry point that allocates nothing and uses the library's
built-in scratch) against aes_sample_build, bit for bit, on two calls in a row, the second
with a smaller input."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _graph(n_rows, n_cols, seed):
    """Degrees from empty rows to a few rows far above every width used below."""
    rng = np.random.default_rng(seed)
    deg = rng.geometric(0.08, size=n_rows).astype(np.int64) - 1
    deg[rng.integers(0, n_rows, size=max(4, n_rows // 500))] = rng.integers(300, 4000, size=max(4, n_rows // 500))
    rowptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(deg, out=rowptr[1:])
    nnz = int(rowptr[-1])
    colidx = rng.integers(0, n_cols, size=nnz).astype(np.int32)
    val = rng.standard_normal(nnz).astype(np.float32)
    return (torch.from_numpy(a).cuda() for a in (rowptr, colidx, val))


def _same(a, b, S):
    assert torch.equal(a.s_rowptr[: a.n_rows + 1], b.s_rowptr[: b.n_rows + 1]), "s_rowptr"
    assert torch.equal(a.s_col[:S], b.s_col[:S]), "s_col"
    assert torch.equal(a.s_val[:S].view(torch.int32), b.s_val[:S].view(torch.int32)), "s_val bits"
    assert torch.equal(a.s_eid[:S], b.s_eid[:S]), "s_eid"
    assert torch.equal(a.row_perm[: a.n_rows], b.row_perm[: b.n_rows]), "row_perm"


def test_noalloc_matches_workspace_entry_point_twice():
    import paper_2503_18427_amd as aes

    assert torch.cuda.is_available()
    # (rows, columns, W): several 1024-row scan blocks and a ragged tail, then a smaller input
    cases = [(70_003, 50_000, 32), (5_001, 3_000, 16)]
    cap0 = None
    buf = None
    for n_rows, n_cols, W in cases:
        print(f"noalloc case n_rows={n_rows} W={W}", flush=True)
        rowptr, colidx, val = _graph(n_rows, n_cols, seed=n_rows)
        ref = aes.aes_sample_build(rowptr, colidx, val, n_cols, W, 0, want_eid=True, want_perm=True)
        torch.cuda.synchronize()
        S = int(ref.s_rowptr[-1].item())
        if buf is None:      # caller-owned outputs, allocated once and reused by the second, smaller call
            cap0 = ref.s_col.numel()
            buf = aes.Plan(n_rows, n_cols, W,
                           torch.full((n_rows + 1,), -7, dtype=torch.int64, device="cuda"),
                           torch.full((cap0,), -7, dtype=torch.int32, device="cuda"),
                           torch.full((cap0,), -7.0, dtype=torch.float32, device="cuda"),
                           torch.full((cap0,), -7, dtype=torch.int64, device="cuda"),
                           torch.full((n_rows,), -7, dtype=torch.int32, device="cuda"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_stats()["allocation.all.allocated"]
        got = aes.aes_sample_build_noalloc(rowptr, colidx, val, n_cols, W, 0, out=buf)
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before, "the call allocated through torch"
        _same(got, ref, S)
    # beyond the built-in scratch: refused on the host, nothing launched
    rp = torch.zeros(2, dtype=torch.int64, device="cuda")
    rc = aes.library().aes_sample_build_noalloc(aes.AES_NOALLOC_MAX_ROWS + 1, 4, 0, rp.data_ptr(), None, None, 4, 0, 0,
                                                rp.data_ptr(), None, None, None, None, None)
    assert rc == -2 and "built-in scratch" in aes.aes_last_error()


def test_noalloc_at_its_row_limit():
    """AES_NOALLOC_MAX_ROWS rows (the whole built-in array is in use), short rows with a few long ones."""
    import paper_2503_18427_amd as aes

    n_rows, n_cols, W = aes.AES_NOALLOC_MAX_ROWS, 1_000_000, 4
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    deg = torch.randint(0, 7, (n_rows,), dtype=torch.int64, device="cuda", generator=g)
    deg[torch.randint(0, n_rows, (64,), device="cuda", generator=g)] = 5000
    rowptr = torch.zeros(n_rows + 1, dtype=torch.int64, device="cuda")
    torch.cumsum(deg, 0, out=rowptr[1:])
    nnz = int(rowptr[-1].item())
    colidx = torch.randint(0, n_cols, (nnz,), dtype=torch.int32, device="cuda", generator=g)
    val = torch.rand(nnz, device="cuda", generator=g)
    print(f"noalloc limit case n_rows={n_rows} nnz={nnz}", flush=True)
    ref = aes.aes_sample_build(rowptr, colidx, val, n_cols, W, 5, want_eid=True, want_perm=True)
    buf = aes.Plan(n_rows, n_cols, W, torch.empty_like(ref.s_rowptr), torch.empty_like(ref.s_col),
                   torch.empty_like(ref.s_val), torch.empty_like(ref.s_eid), torch.empty_like(ref.row_perm))
    got = aes.aes_sample_build_noalloc(rowptr, colidx, val, n_cols, W, 5, out=buf)
    torch.cuda.synchronize()
    _same(got, ref, int(ref.s_rowptr[-1].item()))
