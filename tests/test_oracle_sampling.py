"""Pins of the oracle's sampler: Table 1, Eq. 3 and Algorithm 1's slot layout
(Sec. 3.2-3.3), against hand-worked vectors, band edges and invariants."""
from fractions import Fraction

import numpy as np
import pytest

from conftest import golden_lines
from helpers import random_csr


def _vectors():
    out = []
    for ln in golden_lines("table1_eq3_vectors.txt"):
        a, b, c = [p.split() for p in ln.split("|")]
        out.append((int(a[0]), int(a[1]), int(b[0]), int(b[1]), [int(x) for x in c]))
    return out


@pytest.mark.parametrize("W,nnz,N,cnt,starts", _vectors())
def test_hand_worked_vectors(oracle, W, nnz, N, cnt, starts):
    assert oracle.strategy(nnz, W) == (N, cnt)
    assert [oracle.hash_start(i, nnz, N) for i in range(cnt)] == starts
    assert oracle.row_slots(nnz, W) == N * cnt


def test_band_edges(oracle):
    for ln in golden_lines("table1_band_edges.txt"):
        W, nnz, N, cnt = map(int, ln.split())
        assert oracle.strategy(nnz, W) == (N, cnt), ln


def test_slot_layout_golden(oracle):
    for ln in golden_lines("slot_layout.txt"):
        a, b = ln.split("|")
        W, nnz = map(int, a.split())
        offs = [int(x) for x in b.split()]
        # one row whose element e has column e and value e+0.5: slots reveal offsets
        rowptr = np.array([0, nnz], dtype=np.int64)
        col = np.arange(nnz, dtype=np.int32)
        val = (np.arange(nnz) + 0.5).astype(np.float32)
        s_rowptr, s_col, s_val, s_eid = oracle.sample_build(rowptr, col, val, W, seed=0)
        assert s_rowptr.tolist() == [0, len(offs)]
        assert s_col.tolist() == offs
        assert s_eid.tolist() == offs
        assert s_val.tolist() == [o + 0.5 for o in offs]


def test_bands_by_exact_rational_ratio(oracle):
    """Table 1 evaluated with exact rationals R = row_nnz / W (no integer
    division, no floats) over a dense sweep, including non-power-of-two W."""
    for W in [1, 2, 3, 4, 7, 8, 16, 31, 32, 48, 64, 100, 128, 256, 1000, 1024]:
        probe = set(range(0, 70))
        for k in (1, 2, 36, 54):
            probe.update(range(max(0, k * W - 2), k * W + 3))
        probe.update([100 * W, 12345])
        for nnz in sorted(probe):
            R = Fraction(nnz, W)
            if R <= 1:
                exp = (nnz, 1)
            else:
                c = 4 if R <= 2 else 8 if R <= 36 else 16 if R <= 54 else 32
                exp = (max(1, W // c), min(c, W))
            assert oracle.strategy(nnz, W) == exp, (W, nnz)


def test_power_of_two_width_fills_exactly(oracle):
    for W in [1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024]:
        for nnz in [0, 1, W - 1, W, W + 1, 2 * W, 2 * W + 1, 36 * W + 1, 54 * W + 1, 10 ** 6]:
            if nnz < 0:
                continue
            assert oracle.row_slots(nnz, W) == min(nnz, W)


def test_hash_range_and_seed_zero(oracle):
    rng = np.random.default_rng(0)
    for _ in range(300):
        W = int(rng.choice([4, 16, 32, 64, 256]))
        nnz = int(rng.integers(W + 1, 200 * W))
        N, cnt = oracle.strategy(nnz, W)
        starts = [oracle.hash_start(i, nnz, N) for i in range(cnt)]
        assert starts[0] == 0
        assert all(0 <= s <= nnz - N for s in starts)
        assert starts == [(i * 1429) % (nnz - N + 1) for i in range(cnt)]
    assert oracle.row_offset(0, 12345) == 0


def test_row_offset_definition(oracle):
    """The seed extension: s_r = low 32 bits of seed*(2r+1)*2654435761."""
    for seed, r in [(1, 0), (1, 1), (7, 123456), (2 ** 63 + 5, 2 ** 31), (0xDEADBEEF, 99)]:
        exp = (seed * (2 * r + 1) * 2654435761) & 0xFFFFFFFF
        assert oracle.row_offset(seed, r) == exp


def test_row_offset_invariants(oracle):
    """What the seed extension's offset must satisfy whatever its multiplier is written as (the build's
    own addition to Eq. 3, so nothing printed pins it): it is a product of the seed, the odd number 2r+1
    and an odd constant, reduced mod 2^32.  Hence: seed 0 gives 0 for every row (the paper's Eq. 3);
    an odd seed gives odd offsets that are pairwise distinct over rows (multiplication by an odd number is
    a bijection mod 2^32 and r -> 2r+1 is injective below 2^31); a seed with k trailing zero bits gives
    offsets with exactly k trailing zero bits; and the offset is linear in the seed mod 2^32."""
    rows = list(range(0, 4000)) + [2 ** 20 + 17, 2 ** 30 + 3, 2 ** 31 - 1]
    assert all(oracle.row_offset(0, r) == 0 for r in rows)
    for seed in (1, 3, 0x9E3779B97F4A7C15, 2 ** 64 - 1):
        offs = [oracle.row_offset(seed, r) for r in rows]
        assert all(o % 2 == 1 for o in offs)
        assert len(set(offs)) == len(offs)
    for k in (1, 5, 17, 31):
        for odd in (1, 12345677):
            for r in (0, 1, 99, 2 ** 25 + 1):
                o = oracle.row_offset(odd << k, r)
                assert o % (1 << k) == 0 and (o >> k) % 2 == 1
    assert oracle.row_offset(1 << 32, 7) == 0                   # the seed's high half only shifts the product out
    for a, b, r in ((5, 11, 3), (2 ** 40 + 9, 77, 123456)):
        assert (oracle.row_offset(a, r) + oracle.row_offset(b, r)) % 2 ** 32 == oracle.row_offset(a + b, r)


@pytest.mark.parametrize("W", [1, 4, 16, 32, 48, 64, 256])
@pytest.mark.parametrize("seed", [0, 1234567])
def test_plan_invariants(oracle, W, seed):
    rng = np.random.default_rng(W + seed)
    n = 400
    deg = np.concatenate([rng.integers(0, 3 * W + 2, size=n - 6),
                          [0, W, W + 1, 36 * W + 1, 54 * W + 1, 60 * W]])
    rng.shuffle(deg)
    rowptr, col, val = random_csr(n, 70 * W + 50, deg, rng)
    s_rowptr, s_col, s_val, s_eid = oracle.sample_build(rowptr, col, val, W, seed=seed)
    assert s_rowptr[0] == 0 and s_rowptr[-1] == s_col.size
    for r in range(n):
        nnz = int(deg[r])
        N, cnt = oracle.strategy(nnz, W)
        k0, k1 = int(s_rowptr[r]), int(s_rowptr[r + 1])
        assert k1 - k0 == N * cnt
        if W & (W - 1) == 0:
            assert k1 - k0 == min(nnz, W)
        e = s_eid[k0:k1]
        assert np.all((e >= rowptr[r]) & (e < rowptr[r + 1]))
        assert np.array_equal(s_col[k0:k1], col[e])
        assert np.array_equal(s_val[k0:k1].view(np.uint32), val[e].view(np.uint32))
        if nnz <= W:
            assert np.array_equal(e, np.arange(rowptr[r], rowptr[r + 1]))
        else:
            grid = e.reshape(N, cnt)                  # slot i + j*cnt -> [j, i]
            assert np.all(np.diff(grid, axis=0) == 1)  # N consecutive elements per sample
            assert np.all(grid[0] - rowptr[r] <= nnz - N)
            s_r = oracle.row_offset(seed, r)
            exp = [((i + s_r) * 1429) % (nnz - N + 1) for i in range(cnt)]
            assert (grid[0] - rowptr[r]).tolist() == exp
            if seed == 0:
                assert grid[0, 0] == rowptr[r]


def test_exact_path_is_identity(oracle):
    rng = np.random.default_rng(5)
    deg = rng.integers(0, 90, size=64)
    rowptr, col, val = random_csr(64, 200, deg, rng)
    s_rowptr, s_col, s_val, s_eid = oracle.sample_build(rowptr, col, val, 0)
    assert np.array_equal(s_rowptr, rowptr)
    assert np.array_equal(s_col, col)
    assert np.array_equal(s_eid, np.arange(col.size))


def test_fixed_granularities_golden(oracle):
    for ln in golden_lines("afs_sfs_vectors.txt"):
        a, b, c = [p.split() for p in ln.split("|")]
        mode, W, nnz = map(int, a)
        N, cnt = map(int, b)
        offs = [int(x) for x in c]
        assert oracle.strategy(nnz, W, mode) == (N, cnt)
        rowptr = np.array([0, nnz], dtype=np.int64)
        col = np.arange(nnz, dtype=np.int32)
        val = np.ones(nnz, dtype=np.float32)
        s = oracle.sample_build(rowptr, col, val, W, seed=0, mode=mode)
        assert s[3].tolist() == offs


def test_speed_first_is_row_truncation(oracle):
    """SFS keeps the first W entries of every long row: the product equals the
    exact SpMM of the truncated matrix (scipy), an independent route."""
    import scipy.sparse as sp
    rng = np.random.default_rng(21)
    deg = rng.integers(0, 120, size=150)
    rowptr, col, val = random_csr(150, 300, deg, rng)
    X = rng.standard_normal((300, 10)).astype(np.float32)
    W = 16
    keep = np.concatenate([np.arange(rowptr[r], min(rowptr[r + 1], rowptr[r] + W)) for r in range(150)])
    t_rowptr = np.concatenate([[0], np.cumsum(np.minimum(deg, W))])
    A = sp.csr_matrix((val[keep].astype(np.float64), col[keep], t_rowptr), shape=(150, 300))
    Y = oracle.aes_spmm(rowptr, col, val, W, X, mode=2)
    assert np.allclose(Y, A @ X.astype(np.float64), rtol=0, atol=1e-12)


def test_accuracy_first_invariants(oracle):
    rng = np.random.default_rng(22)
    deg = rng.integers(0, 400, size=120)
    rowptr, col, val = random_csr(120, 500, deg, rng)
    for W in (4, 16, 48):
        s_rowptr, s_col, s_val, s_eid = oracle.sample_build(rowptr, col, val, W, seed=0, mode=1)
        for r in range(120):
            nnz = int(deg[r])
            e = s_eid[s_rowptr[r]:s_rowptr[r + 1]] - rowptr[r]
            if nnz <= W:
                assert e.tolist() == list(range(nnz))
            else:
                assert e.tolist() == [(i * 1429) % nnz for i in range(W)]


def test_sampler_properties_hypothesis(oracle):
    """Property test over (W, row_nnz, seed, mode): slot count, index range, runs of
    N consecutive entries, and agreement of every start with exact-integer Eq. 3."""
    from hypothesis import given, settings, strategies as st

    @settings(max_examples=300, deadline=None)
    @given(W=st.integers(1, 300), nnz=st.integers(0, 40000), seed=st.integers(0, 2 ** 64 - 1),
           mode=st.sampled_from([0, 1, 2]), rid=st.integers(0, 2 ** 31 - 2))
    def check(W, nnz, seed, mode, rid):
        N, cnt = oracle.strategy(nnz, W, mode)
        assert N * cnt == oracle.row_slots(nnz, W, mode)
        if nnz <= W:
            assert (N, cnt) == (nnz, 1)
            return
        assert 1 <= N <= W and 1 <= cnt <= W and N * cnt <= W
        s_r = oracle.row_offset(seed, rid)
        assert s_r == (seed * (2 * rid + 1) * 2654435761) & 0xFFFFFFFF
        for i in (0, cnt // 2, cnt - 1):
            st_i = oracle.hash_start(i + s_r, nnz, N)
            assert st_i == ((i + s_r) * 1429) % (nnz - N + 1)
            assert 0 <= st_i and st_i + N - 1 <= nnz - 1

    check()
