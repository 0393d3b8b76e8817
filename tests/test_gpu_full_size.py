"""Parity at the full benchmark sizes, in the launch configuration bench.py times (default geometry,
nnz hint primed by da_spmm_features, matrix prepared with da_spmm_prepare): every algorithm id on
every named configuration, checked on a seeded sample of rows plus the longest rows, which the
oracle computes one by one."""
import numpy as np
import pytest
import torch

from oracle import reference as orc
from paper_2202_08556_amd import generators as gen

pytestmark = pytest.mark.gpu


def sample_rows(a, nsample=4096, nlong=64, seed=0):
    rng = np.random.Generator(np.random.PCG64(seed))
    rows = rng.choice(a.m, size=min(nsample, a.m), replace=False)
    longest = np.argsort(a.row_lengths())[-nlong:]
    empty = np.nonzero(a.row_lengths() == 0)[0][:64]
    return np.unique(np.concatenate([rows, longest, empty, [0, a.m - 1]])).astype(np.int64)


def check_all(a, B, label):
    from paper_2202_08556_amd import binding as da
    from tests.gpu_util import DeviceProblem
    prob = DeviceProblem(a, B)
    feats = da.da_spmm_features(a.m, prob.N, prob.rowptr)      # as bench.py does: primes the nnz hint
    assert feats["nnz"] == a.nnz
    da.da_spmm_prepare(a.m, a.k, a.nnz, prob.rowptr, prob.colind)   # and builds the EB chunk order
    rows = sample_rows(a)
    c_ref, s_abs = orc.spmm_rows(rows, a.rowptr, a.colind, a.vals, B)
    worst = 0.0
    for algo in range(8):
        print(f"{label} algo={algo}", flush=True)
        c = prob.run(algo)
        ratio = orc.tolerance_ratio(c[rows], c_ref, s_abs)
        assert ratio <= 1.0, f"{label} algo={algo}: tolerance ratio {ratio}"
        assert np.isfinite(c).all(), f"{label} algo={algo}: non-finite output"
        worst = max(worst, ratio)
    da.da_spmm_release(prob.rowptr)
    return worst


@pytest.mark.parametrize("N", [32, 128])
def test_powerlaw_full(N):
    a = gen.powerlaw_csr(seed=gen.config_seed(2))
    check_all(a, gen.dense(a.k, N, "normal", seed=gen.config_seed(2)), f"powerlaw N={N}")


def test_stencil_full():
    a = gen.stencil27_csr(seed=gen.config_seed(3))
    assert a.nnz == 27725560
    check_all(a, gen.dense(a.k, 32, "uniform", seed=gen.config_seed(3)), "stencil N=32")


@pytest.mark.parametrize("N", [8, 64])
def test_skewed_full(N):
    a = gen.skewed_csr(seed=gen.config_seed(4))
    check_all(a, gen.dense(a.k, N, "uniform", seed=gen.config_seed(4)), f"skewed N={N}")


def test_skewed_full_integer_bit_exact():
    # rows of up to 100000 entries split over hundreds of chunks: every atomic / carried partial
    # must land exactly once
    a = gen.integer_twin(gen.skewed_csr(seed=gen.config_seed(4)))
    B = gen.dense_int(a.k, 8, seed=41)
    from tests.gpu_util import DeviceProblem
    prob = DeviceProblem(a, B)
    rows = sample_rows(a)
    c_ref, _ = orc.spmm_rows(rows, a.rowptr, a.colind, a.vals, B, want_abs=False)
    for algo in range(8):
        print(f"skewed int algo={algo}", flush=True)
        c = prob.run(algo)
        assert orc.bit_mismatches(c[rows], c_ref) == 0, f"algo={algo}"


@pytest.mark.parametrize("j,N", [(4, 256), (37, 16), (13, 64), (0, 8)])
def test_sweep_members(j, N):
    a = gen.sweep_csr(j)
    check_all(a, gen.dense(a.k, N, "uniform", seed=a.seed), f"sweep{j} N={N}")


@pytest.mark.parametrize("which", ["powerlaw", "skewed"])
def test_transpose_full(which):
    """da_csr_transpose at the benchmark sizes (13 M / 33 M entries, thousands of sort blocks,
    columns hit a million times): bit for bit against the oracle's stable re-ordering."""
    from tests.test_gpu_transpose_gcn import device_transpose
    a = gen.powerlaw_csr(seed=gen.config_seed(2)) if which == "powerlaw" else gen.skewed_csr(seed=gen.config_seed(4))
    print(f"transpose full {which} nnz={a.nnz}", flush=True)
    ref = orc.csr_transpose(a.rowptr, a.colind, a.vals, a.k)
    got = device_transpose(a)
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
    assert np.array_equal(got[2].view(np.uint32), ref[2].view(np.uint32))
