"""Seeded random small cases through the C ABI against the oracle: shapes, row-length laws, N,
storage orders and leading dimensions drawn at random, every algorithm id, with and without the
per-matrix preparation.  The sizes keep the oracle at milliseconds per case."""
import os

import numpy as np
import pytest
import torch

from oracle import reference as orc
from paper_2202_08556_amd import generators as gen

pytestmark = pytest.mark.gpu


def draw_case(seed):
    rng = np.random.default_rng(seed)
    m = int(rng.integers(1, 3000))
    k = int(rng.integers(1, 3000))
    kind = int(rng.integers(0, 5))
    if kind == 4:                                    # stored rows between long runs of empty rows
        m = int(rng.integers(1000, 30000))
        a = gen.hypersparse_csr(m, k, row_frac=float(rng.uniform(0.002, 0.2)), mean_len=float(rng.uniform(1.0, min(k, 40))),
                                seed=seed)
    elif kind == 0:
        a = gen.uniform_csr(m=m, k=k, mean_len=float(rng.uniform(0.2, min(k, 40))), seed=seed)
    elif kind == 1:
        a = gen.lognormal_csr(m, float(rng.uniform(1.0, min(k, 60))), float(rng.uniform(0.0, 8.0)), seed=seed, k=k,
                              name="lognormal")
    elif kind == 2:
        hi = max(2, min(k, int(rng.integers(2, 2500))))
        a = gen.skewed_csr(m=m, k=k, heavy_frac=float(rng.uniform(0.001, 0.05)), heavy_lo=max(1, hi // 2), heavy_hi=hi,
                           light_mean=float(rng.uniform(0.1, 6.0)), seed=seed)
    else:
        a = gen.powerlaw_csr(m=m, k=k, scale=float(rng.uniform(1.0, 8.0)), max_len=max(1, min(k, 512)), seed=seed)
    N = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 17, 31, 32, 33, 48, 64, 65, 100, 128, 130, 200, 256, 300]))
    return a, N, rng


# DA_TEST_RANDOM_CASES=n widens the default 40 seeds for an occasional longer run
@pytest.mark.parametrize("seed", list(range(9000, 9000 + int(os.environ.get("DA_TEST_RANDOM_CASES", "40")))))
def test_random_case(seed):
    from paper_2202_08556_amd import binding as da
    a, N, rng = draw_case(seed)
    dev = torch.device("cuda:0")
    col_b, col_c = bool(rng.integers(0, 2)) and seed % 3 == 0, bool(rng.integers(0, 2)) and seed % 3 == 0
    ldb = (a.k if col_b else N) + int(rng.integers(0, 4))
    ldc = (a.m if col_c else N) + int(rng.integers(0, 4))
    prepared = seed % 2 == 0
    print(f"random case seed={seed} {a.name} m={a.m} k={a.k} nnz={a.nnz} N={N} colB={col_b} colC={col_c} "
          f"ldb={ldb} ldc={ldc} prepared={prepared}", flush=True)
    Bl = gen.dense(a.k, N, "uniform", seed=seed + 1)
    b_buf = np.zeros((N if col_b else a.k) * ldb, dtype=np.float32)
    orc.dense_view(b_buf, a.k, N, ldb, col_b)[:] = Bl
    c_ref, s_abs = orc.spmm_ex(a.rowptr, a.colind, a.vals, b_buf, a.k, N, ldb, col_b)
    rp, ci, va = (torch.from_numpy(x).to(dev) for x in (a.rowptr, a.colind, a.vals))
    Bd = torch.from_numpy(b_buf).to(dev)
    if prepared:
        da.da_spmm_prepare(a.m, a.k, a.nnz, rp, ci)
    try:
        for algo in range(8):
            c_buf = torch.full(((N if col_c else a.m) * ldc,), float("nan"), device=dev)
            da.da_spmm_ex(a.m, a.k, N, rp, ci, va, Bd, ldb, da.DA_COL_MAJOR if col_b else da.DA_ROW_MAJOR,
                          c_buf, ldc, da.DA_COL_MAJOR if col_c else da.DA_ROW_MAJOR, algo)
            torch.cuda.synchronize()
            got = orc.dense_view(c_buf.cpu().numpy(), a.m, N, ldc, col_c)
            assert orc.tolerance_ratio(got, c_ref, s_abs) <= 1.0, (seed, algo)
            pad = c_buf.cpu().numpy().copy()
            orc.dense_view(pad, a.m, N, ldc, col_c)[:] = 0.0
            assert np.isnan(pad[pad != 0.0]).all()                 # padding between rows / columns untouched
    finally:
        if prepared:
            da.da_spmm_release(rp)


def draw_medium_case(seed):
    rng = np.random.default_rng(seed)
    m = int(rng.integers(20000, 200000))
    kind = int(rng.integers(0, 3))
    if kind == 0:
        a = gen.lognormal_csr(m, float(rng.uniform(8.0, 300.0)), float(rng.choice([0.0, 0.3, 2.0, 8.0])), seed=seed,
                              name="lognormal")
    elif kind == 1:
        a = gen.skewed_csr(m=m, heavy_frac=float(rng.uniform(0.0005, 0.01)), heavy_lo=2000, heavy_hi=min(m, 40000),
                           light_mean=float(rng.uniform(0.5, 20.0)), seed=seed)
    else:
        a = gen.powerlaw_csr(m=m, scale=float(rng.uniform(3.0, 12.0)), max_len=int(rng.choice([512, 4096])), seed=seed)
    return a, int(rng.choice([8, 32, 64, 128])), rng


@pytest.mark.parametrize("seed", list(range(9500, 9510)))
def test_random_medium_case_prepared(seed):
    """Matrices large enough for the chunk schedule, its two segments and the XCD stripes to be in
    use (a few hundred thousand to a few million entries): every id on a prepared matrix against the
    oracle on sampled rows plus the longest rows."""
    from paper_2202_08556_amd import binding as da
    a, N, rng = draw_medium_case(seed)
    print(f"random medium case seed={seed} {a.name} m={a.m} nnz={a.nnz} N={N}", flush=True)
    dev = torch.device("cuda:0")
    B = gen.dense(a.k, N, "uniform", seed=seed + 1)
    rows = np.unique(np.concatenate([rng.integers(0, a.m, size=1500), np.argsort(a.row_lengths())[-32:],
                                     [0, a.m - 1]])).astype(np.int64)
    c_ref, s_abs = orc.spmm_rows(rows, a.rowptr, a.colind, a.vals, B)
    rp, ci, va, Bd = (torch.from_numpy(x).to(dev) for x in (a.rowptr, a.colind, a.vals, B))
    da.da_spmm_features(a.m, N, rp)
    da.da_spmm_prepare(a.m, a.k, a.nnz, rp, ci)
    try:
        for algo in range(8):
            C = torch.full((a.m, N), float("nan"), device=dev)
            da.da_spmm(a.m, a.k, N, rp, ci, va, Bd, C, algo)
            torch.cuda.synchronize()
            c = C.cpu().numpy()
            assert np.isfinite(c).all(), (seed, algo)
            assert orc.tolerance_ratio(c[rows], c_ref, s_abs) <= 1.0, (seed, algo)
    finally:
        da.da_spmm_release(rp)
