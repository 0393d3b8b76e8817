"""Pins for the oracle's transposed product, CSR transpose and graph-convolution layer (the GCN
application of Sec. 6): each check compares with something fixed by mathematics or by an
independent library routine, never with the function itself."""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import reference as orc
from paper_2202_08556_amd import generators as gen


def dense_of(a):
    d = np.zeros((a.m, a.k), dtype=np.float64)
    for i in range(a.m):
        for p in range(a.rowptr[i], a.rowptr[i + 1]):
            d[i, a.colind[p]] += float(a.vals[p])
    return d


def small_cases():
    yield gen.uniform_csr(m=37, k=53, mean_len=5, seed=31)
    yield gen.uniform_csr(m=53, k=29, mean_len=3, seed=32)
    yield gen.powerlaw_csr(m=48, scale=3.0, max_len=40, seed=33)
    yield gen.skewed_csr(m=60, heavy_frac=0.05, heavy_lo=30, heavy_hi=60, seed=34)
    yield gen.fig6a_csr()


# T1 -- the transpose of a tiny matrix, read off its dense form by index loops ------------------
@pytest.mark.parametrize("a", list(small_cases()), ids=lambda a: a.name)
def test_transpose_matches_dense_scan(a):
    d = dense_of(a)
    present = np.zeros((a.m, a.k), dtype=bool)
    for i in range(a.m):
        present[i, a.colind[a.rowptr[i]:a.rowptr[i + 1]]] = True
    rp, ci, va = [0], [], []
    for j in range(a.k):                      # rows of A^T = columns of A
        for i in range(a.m):                  # ascending original row number
            if present[i, j]:
                ci.append(i)
                va.append(np.float32(d[i, j]))
        rp.append(len(ci))
    t_rp, t_ci, t_va = orc.csr_transpose(a.rowptr, a.colind, a.vals, a.k)
    assert t_rp.tolist() == rp and t_ci.tolist() == ci
    assert np.array_equal(t_va, np.array(va, dtype=np.float32))


# T2 -- scipy's CSR -> CSC conversion is the same re-ordering -----------------------------------
@pytest.mark.parametrize("a", [gen.lognormal_csr(3000, 12.0, 3.0, seed=35, name="ln"),
                               gen.powerlaw_csr(m=2048, seed=36)], ids=lambda a: a.name)
def test_transpose_matches_scipy(a):
    s = sp.csr_matrix((a.vals, a.colind, a.rowptr), shape=(a.m, a.k)).tocsc()
    s.sort_indices()
    t_rp, t_ci, t_va = orc.csr_transpose(a.rowptr, a.colind, a.vals, a.k)
    assert np.array_equal(t_rp, s.indptr) and np.array_equal(t_ci, s.indices)
    assert np.array_equal(t_va, s.data)


# T3 -- transposing twice gives the matrix back; a permutation's transpose is its inverse;
#       the 27-point stencil is structurally symmetric ----------------------------------------
def test_transpose_involution_permutation_stencil():
    a = gen.lognormal_csr(1500, 9.0, 2.0, seed=37, name="ln")
    t = orc.csr_transpose(a.rowptr, a.colind, a.vals, a.k)
    b = orc.csr_transpose(t[0], t[1], t[2], a.m)
    assert np.array_equal(b[0], a.rowptr) and np.array_equal(b[1], a.colind) and np.array_equal(b[2], a.vals)

    n = 97
    perm = np.random.default_rng(38).permutation(n).astype(np.int32)
    vals = np.arange(1, n + 1, dtype=np.float32)
    t_rp, t_ci, t_va = orc.csr_transpose(np.arange(n + 1, dtype=np.int32), perm, vals, n)
    inv = np.empty(n, dtype=np.int32)
    inv[perm] = np.arange(n, dtype=np.int32)
    assert np.array_equal(t_rp, np.arange(n + 1)) and np.array_equal(t_ci, inv)
    assert np.array_equal(t_va, vals[inv])

    s = gen.stencil27_csr(6, 5, 7, seed=39)
    t_rp, t_ci, _ = orc.csr_transpose(s.rowptr, s.colind, s.vals, s.k)
    assert np.array_equal(t_rp, s.rowptr) and np.array_equal(t_ci, s.colind)


def test_transpose_empty_rows_columns_and_no_entries():
    rp = np.array([0, 0, 2, 2, 3], dtype=np.int32)                   # 4 x 6, rows 0 and 2 empty
    ci = np.array([5, 1, 1], dtype=np.int32)                         # unsorted inside row 1
    va = np.array([1.0, 2.0, 3.0], dtype=np.float32)
    t_rp, t_ci, t_va = orc.csr_transpose(rp, ci, va, 6)
    assert t_rp.tolist() == [0, 0, 2, 2, 2, 2, 3]
    assert t_ci.tolist() == [1, 3, 1] and t_va.tolist() == [2.0, 3.0, 1.0]
    t_rp, t_ci, t_va = orc.csr_transpose(np.zeros(4, dtype=np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32), 5)
    assert t_rp.tolist() == [0] * 6 and t_ci.size == 0 and t_va.size == 0


# T4 -- A^T.G against the dense fp64 product and against the product with the transposed arrays ---
@pytest.mark.parametrize("a", list(small_cases()), ids=lambda a: a.name)
def test_spmm_transposed_matches_dense(a):
    N = 6
    G = gen.dense(a.m, N, "normal", seed=a.seed + 1)
    d, s = orc.spmm_transposed(a.rowptr, a.colind, a.vals, G, a.k)
    ad = dense_of(a)
    np.testing.assert_allclose(d, ad.T @ G.astype(np.float64), rtol=0, atol=1e-12)
    np.testing.assert_allclose(s, np.abs(ad).T @ np.abs(G.astype(np.float64)), rtol=0, atol=1e-12)
    # a wrong operand order (A.G instead of A^T.G) cannot pass: shapes differ unless square, and
    # for the square cases the dense comparison above already separates them
    t = orc.csr_transpose(a.rowptr, a.colind, a.vals, a.k)
    c, _ = orc.spmm(t[0], t[1], t[2], G)
    np.testing.assert_allclose(d, c, rtol=0, atol=1e-12)


# T5 -- A^T.G is the gradient of <G, A.X> with respect to X: central differences of the forward
#       oracle (exact up to rounding, the function is linear) ------------------------------------
def test_spmm_transposed_is_gradient_of_forward():
    a = gen.uniform_csr(m=21, k=17, mean_len=4, seed=41)
    N = 3
    rng = np.random.default_rng(42)
    X = rng.standard_normal((a.k, N)).astype(np.float32)
    G = rng.standard_normal((a.m, N)).astype(np.float32)
    d, _ = orc.spmm_transposed(a.rowptr, a.colind, a.vals, G, a.k)

    def loss(Xp):
        c, _ = orc.spmm(a.rowptr, a.colind, a.vals, Xp, want_abs=False)
        return float((c * G.astype(np.float64)).sum())

    h = np.float32(0.5)                                   # exactly representable step
    for j in range(a.k):
        for n in range(N):
            Xp, Xm = X.copy(), X.copy()
            Xp[j, n] += h
            Xm[j, n] -= h
            step = float(Xp[j, n]) - float(Xm[j, n])      # the step actually taken in fp32
            assert abs((loss(Xp) - loss(Xm)) / step - d[j, n]) < 1e-9


# T6 -- the layer: forward against dense fp64 algebra, backward against central differences -----
def test_gcn_layer_forward_and_gradients():
    a = gen.uniform_csr(m=14, k=14, mean_len=3, seed=43)
    fin, fout = 5, 4
    rng = np.random.default_rng(44)
    X = rng.standard_normal((a.m, fin))
    W = rng.standard_normal((fin, fout))
    b = rng.standard_normal(fout)
    d_out = rng.standard_normal((a.m, fout))
    out, Z = orc.gcn_layer(a.rowptr, a.colind, a.vals, X, W, b)
    ad = dense_of(a)
    np.testing.assert_allclose(Z, ad @ X @ W + b, rtol=0, atol=1e-12)
    np.testing.assert_allclose(out, np.maximum(ad @ X @ W + b, 0), rtol=0, atol=1e-12)
    assert np.abs(Z).min() > 1e-4                         # no unit sits on the kink of the relu
    dX, dW, db = orc.gcn_layer_backward(a.rowptr, a.colind, a.vals, X, W, Z, d_out)

    def loss(Xp, Wp, bp):
        return float((orc.gcn_layer(a.rowptr, a.colind, a.vals, Xp, Wp, bp)[0] * d_out).sum())

    h = 1e-6
    for arr, grad, which in ((X, dX, 0), (W, dW, 1), (b, db, 2)):
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            args_p, args_m = [X.copy(), W.copy(), b.copy()], [X.copy(), W.copy(), b.copy()]
            args_p[which][idx] += h
            args_m[which][idx] -= h
            fd = (loss(*args_p) - loss(*args_m)) / (2 * h)
            assert abs(fd - grad[idx]) < 1e-6 * max(1.0, abs(grad[idx]))
