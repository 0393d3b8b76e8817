"""Pins for the CPU oracle: every check compares it with something fixed by the paper or by
mathematics, never with itself.  Chosen so that a dropped term, a wrong index (colind*N+n), an
off-by-one in the rowptr range or a transposed operand fails at least one of them."""
import os

import numpy as np
import pytest
import scipy.sparse as sp

from oracle import reference as orc
from paper_2202_08556_amd import generators as gen

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def dense_of(a):
    d = np.zeros((a.m, a.k), dtype=np.float64)
    for i in range(a.m):
        for p in range(a.rowptr[i], a.rowptr[i + 1]):
            d[i, a.colind[p]] += float(a.vals[p])
    return d


def small_cases():
    yield gen.uniform_csr(m=37, k=53, mean_len=5, seed=11), 17
    yield gen.uniform_csr(m=64, k=64, mean_len=9, seed=12), 1
    yield gen.powerlaw_csr(m=48, scale=3.0, max_len=40, seed=13), 8
    yield gen.skewed_csr(m=60, heavy_frac=0.05, heavy_lo=30, heavy_hi=60, seed=14), 5
    yield gen.fig6a_csr(), 3


# P1 -- dense GEMM (BLAS, fp64) on tiny inputs -------------------------------------------------
@pytest.mark.parametrize("case", list(small_cases()), ids=lambda c: f"{c[0].name}-N{c[1]}")
def test_matches_dense_gemm(case):
    a, N = case
    B = gen.dense(a.k, N, "normal", seed=a.seed)
    c, s = orc.spmm(a.rowptr, a.colind, a.vals, B)
    ad = dense_of(a)
    np.testing.assert_allclose(c, ad @ B.astype(np.float64), rtol=0, atol=1e-12)
    np.testing.assert_allclose(s, np.abs(ad) @ np.abs(B.astype(np.float64)), rtol=0, atol=1e-12)


# P9 -- the three-loop model written out literally in pure Python --------------------------------
def test_matches_pure_python_triple_loop():
    a = gen.uniform_csr(m=19, k=23, mean_len=4, seed=21)
    N = 6
    B = gen.dense(a.k, N, "uniform", seed=3)
    y = [[0.0] * N for _ in range(a.m)]
    for m_ in range(a.m):
        for n_ in range(N):
            for p in range(int(a.rowptr[m_]), int(a.rowptr[m_ + 1])):
                y[m_][n_] += float(a.vals[p]) * float(B[int(a.colind[p])][n_])
    c, _ = orc.spmm(a.rowptr, a.colind, a.vals, B)
    np.testing.assert_allclose(c, np.array(y), rtol=0, atol=1e-13)


# P2 -- identity, permutation, diagonal ---------------------------------------------------------
def test_identity_permutation_diagonal():
    k, N = 41, 7
    B = gen.dense(k, N, "normal", seed=5)
    rp = np.arange(k + 1, dtype=np.int32)
    ones = np.ones(k, dtype=np.float32)
    c, s = orc.spmm(rp, np.arange(k, dtype=np.int32), ones, B)
    assert np.array_equal(c, B.astype(np.float64))
    assert np.array_equal(s, np.abs(B.astype(np.float64)))
    pi = np.random.Generator(np.random.PCG64(7)).permutation(k).astype(np.int32)
    c, _ = orc.spmm(rp, pi, ones, B)
    assert np.array_equal(c, B[pi].astype(np.float64))
    d = gen.dense(k, 1, "uniform", seed=8)[:, 0]
    c, _ = orc.spmm(rp, np.arange(k, dtype=np.int32), d, B)
    assert np.array_equal(c, d.astype(np.float64)[:, None] * B.astype(np.float64))


def test_rectangular_and_last_column():
    # one entry in the last column of a wide matrix, one in the first: catches k/N mix-ups
    rp = np.array([0, 1, 2], dtype=np.int32)
    ci = np.array([9, 0], dtype=np.int32)
    v = np.array([2.0, -3.0], dtype=np.float32)
    B = np.arange(10 * 3, dtype=np.float32).reshape(10, 3)
    c, _ = orc.spmm(rp, ci, v, B)
    assert np.array_equal(c, np.array([[54.0, 56.0, 58.0], [0.0, -3.0, -6.0]]))


# P3 -- empty rows, empty matrix, the paper's 6/2/0/3/1 example ---------------------------------
def test_empty_rows_and_empty_matrix():
    B = gen.dense(8, 4, "uniform", seed=1)
    rp = np.array([0, 0, 2, 2, 2, 3, 3], dtype=np.int32)
    ci = np.array([1, 7, 0], dtype=np.int32)
    v = np.array([1.0, 1.0, 2.0], dtype=np.float32)
    c, s = orc.spmm(rp, ci, v, B)
    for r in (0, 2, 3, 5):
        assert np.all(c[r] == 0.0) and np.all(s[r] == 0.0)
    assert np.array_equal(c[1], B[1].astype(np.float64) + B[7].astype(np.float64))
    assert np.array_equal(c[4], 2.0 * B[0].astype(np.float64))
    c, s = orc.spmm(np.zeros(6, dtype=np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32), B)
    assert c.shape == (5, 4) and not c.any() and not s.any()
    c, _ = orc.spmm(np.zeros(1, dtype=np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32), B)
    assert c.shape == (0, 4)


def read_fig6a():
    rows = [l.strip() for l in open(os.path.join(GOLD, "fig6a_row_lengths.txt")) if not l.startswith("#")]
    return [int(x) for x in rows[0].split()], int(rows[1])


def test_fig6a_structure_matches_paper_and_oracle_handles_it():
    lens, width = read_fig6a()
    a = gen.fig6a_csr()
    assert a.row_lengths().tolist() == lens == [6, 2, 0, 3, 1] and width == 4
    B = gen.dense_int(a.k, 5, seed=2)
    c, _ = orc.spmm(a.rowptr, a.colind, a.vals, B)
    assert not c[2].any()
    np.testing.assert_array_equal(c, dense_of(a) @ B.astype(np.float64))


# P4 -- integer-valued inputs are exact; compare with Python big-int arithmetic -----------------
def test_integer_inputs_exact_against_python_ints():
    a = gen.integer_twin(gen.skewed_csr(m=50, heavy_frac=0.06, heavy_lo=35, heavy_hi=50, seed=31))
    N = 4
    B = gen.dense_int(a.k, N, seed=9)
    c, _ = orc.spmm(a.rowptr, a.colind, a.vals, B)
    for i in range(a.m):
        for n in range(N):
            acc = 0
            for p in range(int(a.rowptr[i]), int(a.rowptr[i + 1])):
                acc += int(a.vals[p]) * int(B[a.colind[p], n])
            assert c[i, n] == float(acc)
    assert orc.bit_mismatches(c.astype(np.float32), c) == 0


# P5 -- closed forms ---------------------------------------------------------------------------
def test_sum_of_column_ids():
    a = gen.uniform_csr(m=80, k=97, mean_len=6, seed=41)
    B = np.repeat(np.arange(a.k, dtype=np.float32)[:, None], 3, axis=1) * np.array([1, 2, -1], np.float32)
    c, _ = orc.spmm(a.rowptr, a.colind, np.ones(a.nnz, np.float32), B)
    for i in range(a.m):
        sc = int(a.colind[a.rowptr[i]:a.rowptr[i + 1]].astype(np.int64).sum())
        assert c[i].tolist() == [sc, 2 * sc, -sc]


def test_row_normalised_times_ones():
    a = gen.powerlaw_csr(m=512, scale=4.0, max_len=200, seed=42)   # vals = 1/len as in the graph config
    c, s = orc.spmm(a.rowptr, a.colind, a.vals, np.ones((a.k, 2), np.float32))
    np.testing.assert_allclose(c, 1.0, rtol=0, atol=2e-6)             # fp32 rounding of 1/len only
    np.testing.assert_allclose(s, c, rtol=0, atol=0)


def test_stencil_neighbour_counts():
    nx, ny, nz = 5, 6, 7
    a = gen.stencil27_csr(nx, ny, nz, unit_values=True)
    assert a.nnz == (3 * nx - 2) * (3 * ny - 2) * (3 * nz - 2)
    c, _ = orc.spmm(a.rowptr, a.colind, a.vals, np.ones((a.k, 1), np.float32))
    assert c.sum() == a.nnz
    assert set(np.unique(c).tolist()) == {8.0, 12.0, 18.0, 27.0}
    cnt = c.reshape(nz, ny, nx)
    assert cnt[0, 0, 0] == 8 and cnt[0, 0, 2] == 12 and cnt[0, 2, 2] == 18 and cnt[3, 2, 2] == 27
    assert (c == 27).sum() == (nx - 2) * (ny - 2) * (nz - 2)


# P6 -- linearity, column independence ------------------------------------------------------------
def test_linearity_and_column_independence():
    a = gen.uniform_csr(m=70, k=90, mean_len=7, seed=51)
    B1 = gen.dense_int(a.k, 8, seed=1)
    B2 = gen.dense_int(a.k, 8, seed=2)
    ai = gen.integer_twin(a)
    c1, _ = orc.spmm(ai.rowptr, ai.colind, ai.vals, B1)
    c2, _ = orc.spmm(ai.rowptr, ai.colind, ai.vals, B2)
    c12, _ = orc.spmm(ai.rowptr, ai.colind, ai.vals, B1 + B2)
    assert np.array_equal(c12, c1 + c2)                # integers: exact
    Bf = gen.dense(a.k, 8, "normal", seed=3)
    cf, sf = orc.spmm(a.rowptr, a.colind, a.vals, Bf)
    for n in (0, 3, 7):
        cn, sn = orc.spmm(a.rowptr, a.colind, a.vals, np.ascontiguousarray(Bf[:, n:n + 1]))
        assert np.array_equal(cn[:, 0], cf[:, n]) and np.array_equal(sn[:, 0], sf[:, n])


# P7 -- unsorted columns, duplicate entries -------------------------------------------------------
def test_entry_permutation_and_splitting():
    a = gen.uniform_csr(m=30, k=40, mean_len=8, seed=61)
    B = gen.dense(a.k, 5, "normal", seed=4)
    c0, _ = orc.spmm(a.rowptr, a.colind, a.vals, B)
    rng = np.random.Generator(np.random.PCG64(5))
    ci, v = a.colind.copy(), a.vals.copy()
    for i in range(a.m):
        s, e = a.rowptr[i], a.rowptr[i + 1]
        perm = rng.permutation(e - s)
        ci[s:e], v[s:e] = ci[s:e][perm], v[s:e][perm]
    c1, _ = orc.spmm(a.rowptr, ci, v, B)
    np.testing.assert_allclose(c1, c0, rtol=0, atol=1e-13)
    # split every entry v into v/2 + v/2 (exact in binary): duplicates must add
    rp2 = (a.rowptr.astype(np.int64) * 2).astype(np.int32)
    ci2 = np.repeat(a.colind, 2)
    v2 = np.repeat(a.vals * np.float32(0.5), 2)
    c2, s2 = orc.spmm(rp2, ci2, v2, B)
    np.testing.assert_allclose(c2, c0, rtol=0, atol=1e-13)


# P8 -- an independent library routine ------------------------------------------------------------
@pytest.mark.parametrize("maker,N", [
    (lambda: gen.uniform_csr(m=3000, k=2500, mean_len=8, seed=71), 8),
    (lambda: gen.powerlaw_csr(m=2048, seed=72), 32),
    (lambda: gen.skewed_csr(m=4096, heavy_frac=0.002, heavy_lo=1000, heavy_hi=3000, seed=73), 16),
    (lambda: gen.stencil27_csr(8, 9, 10, seed=74), 5),
])
def test_matches_scipy_csr_product(maker, N):
    a = maker()
    B = gen.dense(a.k, N, "normal", seed=a.seed)
    c, s = orc.spmm(a.rowptr, a.colind, a.vals, B)
    A = sp.csr_matrix((a.vals.astype(np.float64), a.colind, a.rowptr), shape=(a.m, a.k))
    ref = A @ B.astype(np.float64)
    scale = abs(A) @ np.abs(B.astype(np.float64))
    assert np.all(np.abs(c - ref) <= 1e-13 * scale + 1e-300)
    np.testing.assert_allclose(s, scale, rtol=1e-13, atol=0)
    # subset entry point = same rows of the full product
    rows = np.array([0, a.m - 1, a.m // 2, 1, a.m // 3], dtype=np.int64)
    cr, sr = orc.spmm_rows(rows, a.rowptr, a.colind, a.vals, B)
    assert np.array_equal(cr, c[rows]) and np.array_equal(sr, s[rows])


def test_flop_count_matches_per_row_work():
    # Sec. 3.2: row m costs K_(m)*N multiply-adds -> S_abs with unit data counts them
    a = gen.uniform_csr(m=100, k=100, mean_len=5, seed=81)
    N = 3
    _, s = orc.spmm(a.rowptr, a.colind, np.ones(a.nnz, np.float32), np.ones((a.k, N), np.float32))
    assert s.sum() == a.nnz * N
    assert np.array_equal(s[:, 0], a.row_lengths().astype(np.float64))


# features --------------------------------------------------------------------------------------
def test_features_against_numpy_statistics():
    a = gen.skewed_csr(m=2000, heavy_frac=0.01, heavy_lo=200, heavy_hi=900, seed=91)
    f = orc.features(a.rowptr, 32)
    lens = a.row_lengths()
    assert f["rows"] == 2000 and f["nnz"] == a.nnz and f["N"] == 32
    assert f["row_nnz_mean"] == pytest.approx(np.mean(lens), rel=1e-14)
    assert f["row_nnz_std"] == pytest.approx(np.std(lens), rel=1e-12)      # population std
    assert f["row_nnz_max"] == lens.max()
    const = orc.features(np.arange(0, 51, 5), 8)
    assert const["row_nnz_std"] == 0.0 and const["row_nnz_mean"] == 5.0


# conditional reduction (Sec. 4, Fig. 6(e)) ---------------------------------------------------------
def run_sums_scalar(partial, index):
    out = {}
    for pv, ix in zip(partial, index):
        out[ix] = out.get(ix, 0.0) + pv
    return out


@pytest.mark.parametrize("W", [4, 16, 32, 64])
def test_conditional_reduction_valid_lanes_hold_run_sums(W):
    rng = np.random.Generator(np.random.PCG64(100 + W))
    for trial in range(50):
        nruns = int(rng.integers(1, W + 1))
        cuts = np.sort(rng.choice(np.arange(1, W), size=nruns - 1, replace=False)) if nruns > 1 else []
        idx = np.zeros(W, dtype=np.int64)
        for c in cuts:
            idx[c:] += int(rng.integers(1, 4))          # flags increase, possibly skipping rows
        part = rng.integers(-8, 9, size=W).astype(np.float64)
        v, valid = orc.conditional_reduction(part, idx)
        want = run_sums_scalar(part, idx)
        assert valid[0]
        assert valid.sum() == len(want)
        for lane in np.nonzero(valid)[0]:
            assert v[lane] == want[idx[lane]]


def test_conditional_reduction_on_paper_example():
    # worker of 4 lanes walking the 12 stored entries of the 6/2/0/3/1 example, 4 at a time
    lens, W = read_fig6a()
    row_of = np.repeat(np.arange(len(lens)), lens)
    part = np.arange(1.0, 13.0)
    got = {}
    for b in range(0, 12, W):
        v, valid = orc.conditional_reduction(part[b:b + W], row_of[b:b + W])
        for lane in np.nonzero(valid)[0]:
            got[row_of[b + lane]] = got.get(row_of[b + lane], 0.0) + v[lane]   # the cross-worker add
    assert got == {0: 21.0, 1: 15.0, 3: 30.0, 4: 12.0}
    # all lanes same row -> lane 0 holds the total; all different -> nothing moves
    v, valid = orc.conditional_reduction([1, 2, 3, 4], [7, 7, 7, 7])
    assert v[0] == 10 and valid.tolist() == [True, False, False, False]
    v, valid = orc.conditional_reduction([1, 2, 3, 4], [0, 1, 2, 3])
    assert v.tolist() == [1, 2, 3, 4] and valid.all()


# selector figure of merit -----------------------------------------------------------------------
def test_normalized_performance_examples():
    for line in open(os.path.join(GOLD, "normalized_performance_examples.txt")):
        if line.startswith("#") or not line.strip():
            continue
        t0, t1, ch, want = [x.strip() for x in line.split("|")]
        times = [[float(x) for x in t0.split()], [float(x) for x in t1.split()]]
        got = orc.normalized_performance(times, [int(x) for x in ch.split()])
        assert got == pytest.approx(float(want), rel=1e-12)


# acceptance helpers --------------------------------------------------------------------------------
def test_tolerance_ratio_and_bit_mismatches():
    cref = np.array([[1.0, -2.0], [0.0, 4.0]])
    sabs = np.array([[1.0, 2.0], [0.0, 4.0]])
    c = cref.astype(np.float32).copy()
    assert orc.tolerance_ratio(c, cref, sabs) == 0.0
    c[0, 1] += np.float32(2e-5)                       # allowed: 1e-5*2 + 1e-6 = 2.1e-5
    assert 0.9 < orc.tolerance_ratio(c, cref, sabs) <= 1.0
    c[1, 0] = np.float32(2e-6)                        # empty row must be (almost) zero: bound 1e-6
    assert orc.tolerance_ratio(c, cref, sabs) > 1.0
    c[1, 0] = np.nan
    assert orc.tolerance_ratio(c, cref, sabs) == float("inf")
    z = np.array([-0.0, 3.0], dtype=np.float32)
    assert orc.bit_mismatches(z, np.array([0.0, 3.0])) == 0
    assert orc.bit_mismatches(z, np.array([0.0, 3.0000002])) == 1


# storage orders (Sec. 3.3) ---------------------------------------------------------------------
def test_dense_view_and_spmm_ex_against_explicit_index_loops():
    k, N = 5, 3
    a = gen.uniform_csr(m=7, k=k, mean_len=2, seed=95)
    logical = gen.dense_int(k, N, seed=96)
    for col_major, ld in ((False, 3), (False, 5), (True, 5), (True, 8)):
        buf = np.full((N if col_major else k) * ld + 2, 99.0, dtype=np.float32)     # padding = 99
        for r in range(k):
            for n in range(N):
                buf[(r + n * ld) if col_major else (r * ld + n)] = logical[r, n]
        assert np.array_equal(orc.dense_view(buf, k, N, ld, col_major), logical)
        c, _ = orc.spmm_ex(a.rowptr, a.colind, a.vals, buf, k, N, ld, col_major)
        np.testing.assert_array_equal(c, dense_of(a) @ logical.astype(np.float64))
    with pytest.raises(ValueError):
        orc.dense_view(np.zeros(100), k, N, 2, False)
