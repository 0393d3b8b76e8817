"""Statistics and structure of the seeded input generators (CPU only)."""
import numpy as np
import pytest

from paper_2202_08556_amd import generators as gen


def check_structure(a, sorted_unique=True):
    assert a.rowptr.dtype == np.int32 and a.colind.dtype == np.int32 and a.vals.dtype == np.float32
    assert a.rowptr[0] == 0 and a.rowptr[-1] == a.colind.size == a.vals.size
    assert a.rowptr.size == a.m + 1
    assert np.all(np.diff(a.rowptr) >= 0)
    if a.nnz:
        assert a.colind.min() >= 0 and a.colind.max() < a.k
    if sorted_unique and a.nnz > 1:
        d = np.diff(a.colind.astype(np.int64)) > 0
        inner = np.ones(a.nnz - 1, dtype=bool)
        b = a.rowptr[1:-1].astype(np.int64)
        b = b[(b > 0) & (b < a.nnz)]
        inner[b - 1] = False
        assert np.all(d[inner])


def test_uniform_config():
    a = gen.uniform_csr()
    check_structure(a)
    assert a.m == a.k == 4096
    assert 7.7 < a.row_lengths().mean() < 8.3
    assert np.all(np.abs(a.vals) <= 1.0)
    b = gen.uniform_csr()
    assert np.array_equal(a.colind, b.colind) and np.array_equal(a.vals, b.vals)   # seeded
    c = gen.uniform_csr(seed=1001)
    assert not np.array_equal(a.rowptr, c.rowptr)


def test_powerlaw_small_and_degree_law():
    a = gen.powerlaw_csr(m=16384, seed=2001)
    check_structure(a)
    lens = a.row_lengths()
    assert lens.min() >= 1 and lens.max() <= 4096
    # P(len >= d) = scale/d  ->  about 6.8 % of rows have 100 or more entries
    assert 0.05 < np.mean(lens >= 100) < 0.09
    assert 35 < lens.mean() < 65
    np.testing.assert_allclose(a.vals[a.rowptr[:-1]], (1.0 / lens).astype(np.float32))
    # popularity-skewed columns: the most popular 1 % of columns collect far more than 1 % of entries
    cnt = np.sort(np.bincount(a.colind, minlength=a.k))[::-1]
    assert cnt[: a.k // 100].sum() > 0.2 * a.nnz


def test_stencil_closed_form():
    a = gen.stencil27_csr(4, 5, 6)
    check_structure(a)
    assert a.nnz == 10 * 13 * 16
    assert set(np.unique(a.row_lengths()).tolist()) == {8, 12, 18, 27}
    # row 0 touches (0,0,0),(1,0,0),(0,1,0),(1,1,0) and the same in the next plane
    assert a.colind[:8].tolist() == [0, 1, 4, 5, 20, 21, 24, 25]
    assert (3 * 64 - 2) * (3 * 128 - 2) * (3 * 128 - 2) == 27725560


def test_skewed_structure():
    a = gen.skewed_csr(m=32768, heavy_lo=2000, heavy_hi=10000, seed=4001)
    check_structure(a)
    lens = a.row_lengths()
    heavy = lens >= 2000
    assert heavy.sum() == 33
    assert 3.8 < lens[~heavy].mean() < 4.2


@pytest.mark.parametrize("cv", [0.0, 0.5, 5.0])
def test_lognormal_family(cv):
    a = gen.lognormal_csr(20000, 16.0, cv, seed=77)
    check_structure(a)
    lens = a.row_lengths()
    if cv == 0.0:
        assert np.all(lens == 16)
    else:
        assert 0.6 * 16 < lens.mean() < 1.4 * 16
        got = lens.std() / lens.mean()
        assert 0.5 * cv < got < 1.6 * cv


def test_sweep_params_ranges_and_disjoint_seeds():
    seen = set()
    for j in range(64):
        m, mean_len, cv, seed = gen.sweep_params(j)
        assert 2 ** 12 <= m <= 2 ** 20 and 0.0 <= cv <= 20.0
        assert mean_len <= 256.0 and m * mean_len <= 2 ** 26 + 1
        assert (cv == 0.0) == (j % 8 == 0)
        seen.add(seed)
    assert len(seen) == 64
    assert not seen & {gen.sweep_params(j, seed_base=100000)[3] for j in range(256)}


def test_rows_nearly_as_long_as_k():
    a = gen.lognormal_csr(64, 60.0, 0.3, seed=5, k=64)
    check_structure(a)
    assert a.row_lengths().max() <= 64


def test_integer_twin_and_dense():
    a = gen.uniform_csr(m=100, k=100, seed=3)
    t = gen.integer_twin(a)
    assert np.array_equal(t.colind, a.colind)
    assert set(np.unique(t.vals).tolist()) <= {-3.0, -2.0, -1.0, 1.0, 2.0, 3.0}
    B = gen.dense_int(100, 8, seed=1)
    assert B.dtype == np.float32 and B.min() >= -4 and B.max() <= 4 and np.all(B == np.rint(B))
    U = gen.dense(1000, 8, "uniform", seed=1)
    assert U.dtype == np.float32 and U.min() >= -1 and U.max() < 1 and abs(U.mean()) < 0.05
    G = gen.dense(1000, 8, "normal", seed=1)
    assert 0.9 < G.std() < 1.1


def test_rmat_same_size_and_sparsity_different_dispersion():
    stds = []
    for i, (a, b, c) in enumerate(((0.25, 0.25, 0.25), (0.45, 0.22, 0.22), (0.57, 0.19, 0.19))):
        g = gen.rmat_csr(12, 8.0, a, b, c, seed=8100 + i)
        check_structure(g)
        assert g.m == g.k == 4096 and g.nnz == 8 * 4096          # identical size and sparsity
        stds.append(g.row_lengths().std())
    assert stds[0] < stds[1] < stds[2]                           # skewed quadrants -> dispersed rows
    again = gen.rmat_csr(12, 8.0, 0.57, 0.19, 0.19, seed=8102)
    assert np.array_equal(again.colind, g.colind)                 # seeded


def test_reversed_edges_is_the_same_edge_set_reversed():
    a = gen.powerlaw_csr(m=2048, max_len=256, seed=71)
    t = gen.reversed_edges(a)
    assert (t.m, t.k, t.nnz) == (a.k, a.m, a.nnz) and t.rowptr[-1] == a.nnz
    rows_a = np.repeat(np.arange(a.m), np.diff(a.rowptr))
    rows_t = np.repeat(np.arange(t.m), np.diff(t.rowptr))
    fwd = sorted(zip(rows_a.tolist(), a.colind.tolist(), a.vals.tolist()))
    rev = sorted(zip(t.colind.tolist(), rows_t.tolist(), t.vals.tolist()))
    assert fwd == rev
    for i in range(t.m):                                   # columns ascend inside every row
        seg = t.colind[t.rowptr[i]:t.rowptr[i + 1]]
        assert np.all(np.diff(seg) > 0)
    # popular columns become rows longer than any row of the original (capped at 256 entries)
    assert t.row_lengths().max() > 2 * a.row_lengths().max()


def test_hypersparse_has_few_stored_rows_between_long_empty_runs():
    a = gen.hypersparse_csr(200_000, 5000, row_frac=0.005, mean_len=40.0, seed=11)
    check_structure(a)
    lens = a.row_lengths()
    stored = np.nonzero(lens)[0]
    assert stored.size == 1000 and lens[stored].min() >= 1
    assert 30 < lens[stored].mean() < 50
    assert np.diff(stored).max() > 500                      # runs of hundreds of empty rows
    again = gen.hypersparse_csr(200_000, 5000, row_frac=0.005, mean_len=40.0, seed=11)
    assert np.array_equal(again.rowptr, a.rowptr) and np.array_equal(again.colind, a.colind)
