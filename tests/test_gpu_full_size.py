"""Parity at the full benchmark sizes, in the launch configuration bench.py times (default geometry,
nnz hint primed by da_spmm_features, matrix prepared with da_spmm_prepare): every algorithm id on
every named configuration, every element of C against the fp64 oracle (the definition of Sec. 3.1
over all rows; all named configurations have nnz * N below 2^31, which the oracle finishes in a
fraction of a second).  The integer twin is compared bit for bit over the whole of C, unprepared
and prepared."""
import numpy as np
import pytest
import torch

from oracle import reference as orc
from paper_2202_08556_amd import generators as gen

pytestmark = pytest.mark.gpu


def whole_c_ratio(c, c_ref, s_abs, block=65536):
    """tolerance_ratio over the whole of C, taken in row blocks to bound the temporaries."""
    worst = 0.0
    for r0 in range(0, c.shape[0], block):
        worst = max(worst, orc.tolerance_ratio(c[r0:r0 + block], c_ref[r0:r0 + block], s_abs[r0:r0 + block]))
    return worst


def check_all(a, B, label, prepare=True):
    from paper_2202_08556_amd import binding as da
    from tests.gpu_util import DeviceProblem
    prob = DeviceProblem(a, B)
    feats = da.da_spmm_features(a.m, prob.N, prob.rowptr)      # as bench.py does: primes the nnz hint
    assert feats["nnz"] == a.nnz
    if prepare:
        da.da_spmm_prepare(a.m, a.k, a.nnz, prob.rowptr, prob.colind)   # and builds the EB chunk order
    c_ref, s_abs = orc.spmm(a.rowptr, a.colind, a.vals, B)
    worst = 0.0
    try:
        for algo in range(8):
            print(f"{label} algo={algo}", flush=True)
            ratio = whole_c_ratio(prob.run(algo), c_ref, s_abs)
            assert ratio <= 1.0, f"{label} algo={algo}: tolerance ratio {ratio}"
            worst = max(worst, ratio)
    finally:
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


@pytest.mark.parametrize("prepare", [False, True], ids=["unprepared", "prepared"])
def test_skewed_full_integer_bit_exact(prepare):
    # rows of up to 100000 entries split over hundreds of chunks: every atomic / carried partial
    # must land exactly once, in storage order of the chunks and in the scheduled, striped order
    from paper_2202_08556_amd import binding as da
    from tests.gpu_util import DeviceProblem
    a = gen.integer_twin(gen.skewed_csr(seed=gen.config_seed(4)))
    B = gen.dense_int(a.k, 8, seed=41)
    prob = DeviceProblem(a, B)
    c_ref, _ = orc.spmm(a.rowptr, a.colind, a.vals, B, want_abs=False)
    if prepare:
        da.da_spmm_features(a.m, prob.N, prob.rowptr)
        da.da_spmm_prepare(a.m, a.k, a.nnz, prob.rowptr, prob.colind)
    try:
        for algo in range(8):
            print(f"skewed int prepare={prepare} algo={algo}", flush=True)
            assert orc.bit_mismatches(prob.run(algo), c_ref) == 0, f"algo={algo}"
    finally:
        da.da_spmm_release(prob.rowptr)


@pytest.mark.parametrize("N", [32, 128])
def test_powerlaw_full_integer_bit_exact(N):
    from paper_2202_08556_amd import binding as da
    from tests.gpu_util import DeviceProblem
    a = gen.integer_twin(gen.powerlaw_csr(seed=gen.config_seed(2)))
    B = gen.dense_int(a.k, N, seed=43)
    prob = DeviceProblem(a, B)
    c_ref, _ = orc.spmm(a.rowptr, a.colind, a.vals, B, want_abs=False)
    da.da_spmm_features(a.m, prob.N, prob.rowptr)
    da.da_spmm_prepare(a.m, a.k, a.nnz, prob.rowptr, prob.colind)
    try:
        for algo in range(8):
            print(f"powerlaw int N={N} algo={algo}", flush=True)
            assert orc.bit_mismatches(prob.run(algo), c_ref) == 0, f"algo={algo}"
    finally:
        da.da_spmm_release(prob.rowptr)


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
