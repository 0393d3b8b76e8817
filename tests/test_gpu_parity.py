"""Parity of the HIP path with the CPU oracle, element by element, through the C ABI.

Tolerance (fp32 result against the fp64 definition): |C - C_ref| <= 1e-5 * (|A|.|B|)_ij + 1e-6.
Integer-valued inputs must match bit for bit (after mapping -0 to +0)."""
import numpy as np
import pytest
import torch

from oracle import reference as orc
from paper_2202_08556_amd import generators as gen

pytestmark = pytest.mark.gpu

ALGOS = list(range(8))


def hypersparse(m=120000, k=4000, seed=31):
    """Most rows empty, in runs from one to hundreds of rows, between short rows: a chunk of stored
    entries then spans many rows with long gaps (the EB row walk has to skip the runs)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    lens = np.zeros(m, np.int64)
    pos = np.cumsum(rng.choice([1, 2, 3, 5, 9, 40, 300], size=m))      # gaps of every kind
    pos = pos[pos < m]
    lens[pos] = rng.integers(1, 30, size=len(pos))
    rowptr, colind = gen.csr_from_lens(rng, lens, k)
    vals = rng.uniform(-1.0, 1.0, size=len(colind)).astype(np.float32)
    return gen.CSR(m, k, rowptr.astype(np.int32), colind.astype(np.int32), vals, "hypersparse", seed)


def problems():
    """Sizes the oracle finishes in well under a second each, spanning several tiles and chunks,
    with ragged tails in m, nnz and N."""
    yield "fig6a", gen.fig6a_csr(), [1, 3, 4, 8]
    yield "uniform", gen.uniform_csr(seed=1000), [8, 33]
    yield "uniform_ragged", gen.uniform_csr(m=1237, k=911, mean_len=11, seed=7), [1, 2, 6, 20, 64, 100]
    yield "powerlaw", gen.powerlaw_csr(m=8192, seed=2001), [32, 128]
    yield "stencil", gen.stencil27_csr(12, 13, 14, seed=3001), [32, 7]
    yield "skewed", gen.skewed_csr(m=16384, heavy_lo=3000, heavy_hi=9000, seed=4001), [8, 64]
    yield "lognormal_cv4", gen.lognormal_csr(5000, 24.0, 4.0, seed=5100), [16, 256, 260]
    yield "const_rows", gen.lognormal_csr(3000, 64.0, 0.0, seed=5101), [4, 48]
    yield "one_long_row", gen.skewed_csr(m=64, k=40000, heavy_frac=0.02, heavy_lo=30000,
                                         heavy_hi=30000, light_mean=0.5, seed=9), [8, 12]
    yield "rmat", gen.rmat_csr(12, 16.0, 0.57, 0.19, 0.19, seed=8102), [4, 32]
    yield "hypersparse", hypersparse(), [8, 64, 128]
    # wide B: several column tiles with a ragged last one (520 = 2*256 + 8; 1030 is not a multiple of 4)
    yield "wide_N", gen.skewed_csr(m=900, k=700, heavy_frac=0.01, heavy_lo=300, heavy_hi=600, seed=10), [520, 1030]


CASES = [(name, a, N) for name, a, Ns in problems() for N in Ns]


@pytest.fixture(scope="module")
def gpu():
    from tests.gpu_util import DeviceProblem
    return DeviceProblem


@pytest.mark.parametrize("name,a,N", CASES, ids=[f"{c[0]}-N{c[2]}" for c in CASES])
def test_all_algorithms_match_oracle(gpu, name, a, N):
    B = gen.dense(a.k, N, "normal" if "power" in name else "uniform", seed=a.seed + N)
    c_ref, s_abs = orc.spmm(a.rowptr, a.colind, a.vals, B)
    prob = gpu(a, B)
    for algo in ALGOS:
        print(f"case {name} N={N} algo={algo}", flush=True)
        c = prob.run(algo)
        ratio = orc.tolerance_ratio(c, c_ref, s_abs)
        assert ratio <= 1.0, f"{name} N={N} algo={algo}: tolerance ratio {ratio}"
        empty = a.row_lengths() == 0
        assert np.all(c[empty].view(np.uint32) == 0), "rows without entries must be +0"


@pytest.mark.parametrize("name,a,N", CASES, ids=[f"{c[0]}-N{c[2]}" for c in CASES])
def test_integer_inputs_bit_exact(gpu, name, a, N):
    ai = gen.integer_twin(a)
    B = gen.dense_int(a.k, N, seed=a.seed + N)
    c_ref, _ = orc.spmm(ai.rowptr, ai.colind, ai.vals, B, want_abs=False)
    prob = gpu(ai, B)
    for algo in ALGOS:
        print(f"int case {name} N={N} algo={algo}", flush=True)
        for rep in range(2):                      # atomics: order may vary, bits may not
            c = prob.run(algo)
            assert orc.bit_mismatches(c, c_ref) == 0, f"{name} N={N} algo={algo} rep={rep}"


def test_unsorted_columns_and_duplicates(gpu):
    a = gen.uniform_csr(m=700, k=500, mean_len=9, seed=21)
    rng = np.random.Generator(np.random.PCG64(3))
    ci, v = a.colind.copy(), a.vals.copy()
    for i in range(a.m):
        s, e = a.rowptr[i], a.rowptr[i + 1]
        p = rng.permutation(e - s)
        ci[s:e], v[s:e] = ci[s:e][p], v[s:e][p]
    # duplicate every entry (halved values) so that repeated (i,j) must add
    dup = gen.CSR(a.m, a.k, (a.rowptr.astype(np.int64) * 2).astype(np.int32), np.repeat(ci, 2),
                  np.repeat(v * np.float32(0.5), 2), "dup", a.seed)
    B = gen.dense(a.k, 12, "uniform", seed=4)
    c_ref, s_abs = orc.spmm(dup.rowptr, dup.colind, dup.vals, B)
    prob = gpu(dup, B)
    for algo in ALGOS:
        assert orc.tolerance_ratio(prob.run(algo), c_ref, s_abs) <= 1.0


def test_degenerate_shapes(gpu):
    from paper_2202_08556_amd import binding as da
    dev = torch.device("cuda:0")
    # nnz == 0: C must be zero-filled by every algorithm
    m, k, N = 300, 50, 24
    a = gen.CSR(m, k, np.zeros(m + 1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32), "empty", 0)
    B = gen.dense(k, N, "uniform", seed=1)
    prob = gpu(a, B)
    for algo in ALGOS:
        assert not prob.run(algo).any()
    # a single row and a single column
    a = gen.uniform_csr(m=1, k=777, mean_len=300, seed=5)
    B = gen.dense(a.k, 1, "uniform", seed=6)
    c_ref, s_abs = orc.spmm(a.rowptr, a.colind, a.vals, B)
    prob = gpu(a, B)
    for algo in ALGOS:
        assert orc.tolerance_ratio(prob.run(algo), c_ref, s_abs) <= 1.0
    # m == 0 and N == 0 are no-ops that leave C untouched
    C = torch.full((4, 4), 7.0, device=dev)
    z = torch.zeros(1, dtype=torch.int32, device=dev)
    da.da_spmm(0, 4, 4, z, z, C, C, C, 0)
    da.da_spmm(4, 4, 0, z, z, C, C, C, 4)
    torch.cuda.synchronize()
    assert torch.all(C == 7.0)
    # unaligned B / C base (offset by one float) forces the scalar-width path
    a = gen.uniform_csr(m=500, k=400, mean_len=7, seed=8)
    N = 8
    Bh = gen.dense(a.k, N, "uniform", seed=9)
    c_ref, s_abs = orc.spmm(a.rowptr, a.colind, a.vals, Bh)
    rp, ci, va = (torch.from_numpy(x).to(dev) for x in (a.rowptr, a.colind, a.vals))
    Bbuf = torch.zeros(a.k * N + 1, device=dev)
    Bbuf[1:] = torch.from_numpy(Bh).to(dev).reshape(-1)
    Cbuf = torch.full((a.m * N + 1,), float("nan"), device=dev)
    for algo in ALGOS:
        da.da_spmm(a.m, a.k, N, rp, ci, va, Bbuf.data_ptr() + 4, Cbuf.data_ptr() + 4, algo)
        torch.cuda.synchronize()
        c = Cbuf[1:].reshape(a.m, N).cpu().numpy()
        assert orc.tolerance_ratio(c, c_ref, s_abs) <= 1.0


def test_features_match_oracle(gpu):
    from paper_2202_08556_amd import binding as da
    for a in (gen.skewed_csr(m=16384, heavy_lo=3000, heavy_hi=9000, seed=4001),
              gen.lognormal_csr(5000, 24.0, 0.0, seed=1), gen.fig6a_csr()):
        rp = torch.from_numpy(a.rowptr).to("cuda:0")
        got = da.da_spmm_features(a.m, 32, rp)
        want = orc.features(a.rowptr, 32)
        assert got["rows"] == want["rows"] and got["nnz"] == want["nnz"] and got["N"] == 32
        assert got["row_nnz_max"] == want["row_nnz_max"]
        assert got["row_nnz_mean"] == pytest.approx(want["row_nnz_mean"], rel=1e-14)
        assert got["row_nnz_std"] == pytest.approx(want["row_nnz_std"], rel=1e-9, abs=1e-12)
        assert 0 <= da.da_spmm_select(got) < 8


def test_side_stream_and_prepared_call(gpu):
    """The stream argument is honoured and the pre-marshalled call gives the same result."""
    from paper_2202_08556_amd import binding as da
    a = gen.lognormal_csr(4000, 12.0, 2.0, seed=77)
    N = 40
    B = gen.dense(a.k, N, "uniform", seed=78)
    c_ref, s_abs = orc.spmm(a.rowptr, a.colind, a.vals, B)
    prob = gpu(a, B)
    side = torch.cuda.Stream()
    for algo in ALGOS:
        C = torch.full((a.m, N), float("nan"), device=prob.B.device)
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            run = da.PreparedSpmm(a.m, a.k, N, prob.rowptr, prob.colind, prob.vals, prob.B, C)
            run(algo)
        side.synchronize()
        assert orc.tolerance_ratio(C.cpu().numpy(), c_ref, s_abs) <= 1.0
        C.fill_(float("nan"))
        torch.cuda.synchronize()
        da.da_spmm(a.m, a.k, N, prob.rowptr, prob.colind, prob.vals, prob.B, C, algo, stream=side)
        side.synchronize()
        assert orc.tolerance_ratio(C.cpu().numpy(), c_ref, s_abs) <= 1.0


def test_tuning_overrides_are_validated_and_correct(gpu, monkeypatch):
    """Geometry overrides used for measurement runs: valid ones give the same C, invalid ones an error."""
    import os
    import subprocess
    import sys
    code = r"""
import os, sys, numpy as np, torch
sys.path.insert(0, os.getcwd())
from oracle import reference as orc
from paper_2202_08556_amd import binding as da, generators as gen
a = gen.lognormal_csr(3000, 20.0, 3.0, seed=5); N = 128
B = gen.dense(a.k, N, "uniform", seed=6)
c_ref, s_abs = orc.spmm(a.rowptr, a.colind, a.vals, B)
dev = torch.device("cuda:0")
rp, ci, va, Bd = (torch.from_numpy(x).to(dev) for x in (a.rowptr, a.colind, a.vals, B))
for env, algos, ok in [(dict(G="8", PIN="1"), (0, 1, 4, 5), True), (dict(G="16", PIN="1", CHUNK="64"), (0, 4), True),
                       (dict(V="1", G="64"), (0, 4), True), (dict(NV="2"), (2, 3, 6, 7), True),
                       (dict(G="8"), (1, 5), True), (dict(G="16"), (1, 5), True), (dict(G="32"), (1, 5), True),
                       (dict(G="3"), (0,), False), (dict(V="2"), (0,), False), (dict(G="64", V="1"), (1,), False)]:
    for k in ("V", "G", "NV", "CHUNK", "PIN"):
        os.environ.pop("DA_SPMM_" + k, None)
    for k, v in env.items():
        os.environ["DA_SPMM_" + k] = v
    for algo in algos:
        C = torch.full((a.m, N), float("nan"), device=dev)
        st = da.da_spmm_status(a.m, a.k, N, rp, ci, va, Bd, C, algo)
        torch.cuda.synchronize()
        if ok:
            assert st == 0, (env, algo, st, da.da_spmm_last_error())
            r = orc.tolerance_ratio(C.cpu().numpy(), c_ref, s_abs)
            assert r <= 1.0, (env, algo, r)
        else:
            assert st == da.DA_ERR_UNSUPPORTED, (env, algo, st)
# column tiles pinned to XCDs together with the chunk order of a prepared matrix (stripes dealt
# to the XCDs that share a tile), on a matrix with enough chunks for several stripes
a = gen.skewed_csr(m=20000, k=15000, heavy_frac=0.01, heavy_lo=4000, heavy_hi=9000, seed=12); N = 128
B = gen.dense(a.k, N, "uniform", seed=7)
c_ref, s_abs = orc.spmm(a.rowptr, a.colind, a.vals, B)
rp, ci, va, Bd = (torch.from_numpy(x).to(dev) for x in (a.rowptr, a.colind, a.vals, B))
da.da_spmm_features(a.m, N, rp)
da.da_spmm_prepare(a.m, a.k, a.nnz, rp, ci)
for env in (dict(G="16", PIN="1"), dict(G="8", PIN="1"), dict(G="16", PIN="1", CHUNK="64", STRIPE="16"), dict(G="4", PIN="1")):
    for k in ("V", "G", "NV", "CHUNK", "PIN", "STRIPE"):
        os.environ.pop("DA_SPMM_" + k, None)
    for k, v in env.items():
        os.environ["DA_SPMM_" + k] = v
    for algo in (4, 5):
        C = torch.full((a.m, N), float("nan"), device=dev)
        st = da.da_spmm_status(a.m, a.k, N, rp, ci, va, Bd, C, algo)
        torch.cuda.synchronize()
        assert st == 0, (env, algo, st, da.da_spmm_last_error())
        r = orc.tolerance_ratio(C.cpu().numpy(), c_ref, s_abs)
        assert r <= 1.0, ("prepared", env, algo, r)
da.da_spmm_release()
print("overrides ok")
"""
    env = dict(os.environ, DA_SPMM_TUNE="1")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, "-c", code], cwd=root, env=env, capture_output=True, text=True, timeout=240)
    assert res.returncode == 0 and "overrides ok" in res.stdout, res.stdout + res.stderr


@pytest.mark.parametrize("prepared", [False, True], ids=["plain", "prepared"])
def test_calls_can_be_captured_in_a_hip_graph(gpu, prepared):
    """da_spmm only enqueues kernels (no allocation, no synchronisation, no memset nodes), so a
    sequence of calls can be captured once and replayed; every replay must reproduce the eager
    result, with eager work and synchronisations between the replays.  Also with a prepared matrix
    large enough for the chunk schedule and its XCD stripes to be in use."""
    from paper_2202_08556_amd import binding as da
    a = gen.skewed_csr(m=16384, heavy_lo=3000, heavy_hi=9000, seed=4001) if prepared else gen.uniform_csr(seed=1000)
    N = 8
    B = gen.dense(a.k, N, "uniform", seed=1000)
    c_ref, s_abs = orc.spmm(a.rowptr, a.colind, a.vals, B)
    prob = gpu(a, B)
    da.da_spmm_features(a.m, N, prob.rowptr)
    if prepared:
        da.da_spmm_prepare(a.m, a.k, a.nnz, prob.rowptr, prob.colind)
    dev = prob.B.device
    outs = [torch.full((a.m, N), float("nan"), device=dev) for _ in range(8)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for algo in ALGOS:                                   # warm-up outside capture
            da.da_spmm(a.m, a.k, N, prob.rowptr, prob.colind, prob.vals, prob.B, outs[algo], algo)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for algo in ALGOS:
            da.da_spmm(a.m, a.k, N, prob.rowptr, prob.colind, prob.vals, prob.B, outs[algo], algo)
    for replay in range(3):
        for o in outs:
            o.fill_(float("nan"))                            # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for algo in ALGOS:
            r = orc.tolerance_ratio(outs[algo].cpu().numpy(), c_ref, s_abs)
            assert r <= 1.0, f"replay {replay} algo {algo}: {r}"
    if prepared:
        da.da_spmm_release(prob.rowptr)


@pytest.mark.parametrize("b_col,c_col", [(False, False), (True, False), (False, True), (True, True)])
def test_storage_orders_and_leading_dimensions(gpu, b_col, c_col):
    """da_spmm_ex: every algorithm id with B and C row- or column-major and padded leading
    dimensions; padding of C must stay untouched."""
    from paper_2202_08556_amd import binding as da
    dev = torch.device("cuda:0")
    a = gen.skewed_csr(m=1500, k=1100, heavy_frac=0.004, heavy_lo=400, heavy_hi=900, seed=31)
    rp, ci, va = (torch.from_numpy(x).to(dev) for x in (a.rowptr, a.colind, a.vals))
    for N, pad in ((8, 0), (36, 4), (5, 3)):
        ldb = (a.k if b_col else N) + pad
        ldc = (a.m if c_col else N) + pad
        logical = gen.dense(a.k, N, "uniform", seed=32 + N)
        b_host = np.full((N if b_col else a.k) * ldb, 7.0, dtype=np.float32)
        orc.dense_view(b_host, a.k, N, ldb, b_col)[...] = logical
        c_ref, s_abs = orc.spmm_ex(a.rowptr, a.colind, a.vals, b_host, a.k, N, ldb, b_col)
        Bd = torch.from_numpy(b_host).to(dev)
        for algo in ALGOS:
            print(f"layouts B{'C' if b_col else 'R'} C{'C' if c_col else 'R'} N={N} algo={algo}", flush=True)
            Cd = torch.full(((N if c_col else a.m) * ldc,), -5.0, device=dev)
            da.da_spmm_ex(a.m, a.k, N, rp, ci, va, Bd, ldb, int(b_col), Cd, ldc, int(c_col), algo)
            torch.cuda.synchronize()
            c_host = Cd.cpu().numpy()
            got = orc.dense_view(c_host, a.m, N, ldc, c_col)
            assert orc.tolerance_ratio(got, c_ref, s_abs) <= 1.0
            mask = np.ones(c_host.size, dtype=bool)
            idx = np.arange(c_host.size).reshape(-1)
            orc.dense_view(mask, a.m, N, ldc, c_col)[...] = False
            assert np.all(c_host[mask] == -5.0), "padding of C was written"


def test_validate_catches_malformed_csr_and_debug_switch_guards_the_product(monkeypatch):
    """da_csr_validate names each kind of violation; with DA_SPMM_DEBUG_VALIDATE=1 the product and
    the transpose refuse malformed arrays before any of their kernels is launched."""
    from paper_2202_08556_amd import binding as da
    dev = torch.device("cuda:0")
    a = gen.uniform_csr(m=300, k=200, mean_len=6, seed=61)
    nnz = int(a.colind.size)
    up = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dev)
    rp, ci, va = up(a.rowptr), up(a.colind), up(a.vals)
    da.da_csr_validate(a.m, a.k, nnz, rp, ci)
    da.da_csr_validate(a.m, a.k, -1, rp, ci)
    bad = da.DA_ERR_INVALID_ARG

    def status_and_text(*args):
        st = da.da_csr_validate_status(*args)
        return st, da.da_spmm_last_error()

    assert status_and_text(a.m, a.k, nnz + 1, rp, ci) == (bad, "malformed CSR: rowptr[m] differs from nnz")
    shifted = a.rowptr.copy(); shifted[0] = 1
    assert status_and_text(a.m, a.k, nnz, up(shifted), ci)[1] == "malformed CSR: rowptr[0] != 0"
    swapped = a.rowptr.copy(); swapped[[100, 101]] = swapped[[101, 100]]
    assert swapped[100] > swapped[101]
    assert status_and_text(a.m, a.k, nnz, up(swapped), ci)[1] == "malformed CSR: rowptr decreases"
    for wrong in (a.k, -1, 2 ** 31 - 1):
        c2 = a.colind.copy(); c2[nnz // 2] = wrong
        assert status_and_text(a.m, a.k, nnz, rp, up(c2)) == (bad, "malformed CSR: column index outside [0, k)")
    assert status_and_text(a.m, a.k - 1, nnz, rp, ci)[0] == (bad if a.colind.max() == a.k - 1 else da.DA_OK)

    # the switch: same malformed arrays through the product and the transpose
    monkeypatch.setenv("DA_SPMM_DEBUG_VALIDATE", "1")
    N = 8
    B = torch.zeros((a.k, N), device=dev)
    C = torch.zeros((a.m, N), device=dev)
    c2 = a.colind.copy(); c2[3] = a.k + 5
    assert da.da_spmm_status(a.m, a.k, N, rp, up(c2), va, B, C, da.DA_EB_RM_SR) == bad
    assert da.da_spmm_status(a.m, a.k, N, up(swapped), ci, va, B, C, da.DA_RB_RM_SR) == bad
    t = (torch.zeros(a.k + 1, dtype=torch.int32, device=dev), torch.zeros(nnz, dtype=torch.int32, device=dev),
         torch.zeros(nnz, dtype=torch.float32, device=dev))
    nbytes = da.da_csr_transpose_workspace(a.m, a.k, nnz)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    assert da.da_csr_transpose_status(a.m, a.k, nnz, rp, up(c2), va, *t, ws, nbytes) == bad
    # well-formed arrays still run, and give the right answer, with the switch on
    Bn = gen.dense(a.k, N, "uniform", seed=5)
    C = torch.full((a.m, N), float("nan"), device=dev)
    assert da.da_spmm_status(a.m, a.k, N, rp, ci, va, up(Bn), C, da.DA_EB_RM_PR) == da.DA_OK
    torch.cuda.synchronize()
    c_ref, s_abs = orc.spmm(a.rowptr, a.colind, a.vals, Bn)
    assert orc.tolerance_ratio(C.cpu().numpy(), c_ref, s_abs) <= 1.0


def test_wide_address_kernels_match_oracle(gpu, monkeypatch):
    """Operands beyond 4 GiB (or k >= 2^24) take kernels with 64-bit gather addresses; the switch
    DA_SPMM_WIDE=1 forces them on small inputs so that they are checked here too."""
    monkeypatch.setenv("DA_SPMM_WIDE", "1")
    for a, N in ((gen.skewed_csr(m=16384, heavy_lo=3000, heavy_hi=9000, seed=4001), 64),
                 (gen.uniform_csr(m=1237, k=911, mean_len=11, seed=7), 20),
                 (gen.powerlaw_csr(m=8192, seed=2001), 128)):
        B = gen.dense(a.k, N, "uniform", seed=a.seed + N)
        c_ref, s_abs = orc.spmm(a.rowptr, a.colind, a.vals, B)
        prob = gpu(a, B)
        for algo in ALGOS:
            print(f"wide case {a.name} N={N} algo={algo}", flush=True)
            assert orc.tolerance_ratio(prob.run(algo), c_ref, s_abs) <= 1.0, (a.name, N, algo)


def test_concurrent_host_threads_on_their_own_streams(gpu):
    """Four host threads call the library at once, each on its own stream and matrix (one of them
    preparing and releasing its matrix between calls): every result matches the oracle."""
    import threading
    from paper_2202_08556_amd import binding as da
    dev = torch.device("cuda:0")
    jobs = []
    for t, (a, N) in enumerate([(gen.lognormal_csr(6000, 30.0, 3.0, seed=90), 32),
                                (gen.powerlaw_csr(m=8192, seed=91), 128),
                                (gen.uniform_csr(m=5000, k=3000, mean_len=9, seed=92), 8),
                                (gen.skewed_csr(m=8192, heavy_lo=2000, heavy_hi=6000, seed=93), 64)]):
        Bh = gen.dense(a.k, N, "uniform", seed=94 + t)
        c_ref, s_abs = orc.spmm(a.rowptr, a.colind, a.vals, Bh)
        rp, ci, va, Bd = (torch.from_numpy(x).to(dev) for x in (a.rowptr, a.colind, a.vals, Bh))
        jobs.append(dict(a=a, N=N, rp=rp, ci=ci, va=va, B=Bd, C=torch.empty((a.m, N), device=dev),
                         ref=c_ref, s_abs=s_abs, stream=torch.cuda.Stream(), worst=0.0, error=None))
    torch.cuda.synchronize()

    def work(t, job):
        try:
            a, N = job["a"], job["N"]
            for it in range(24):
                algo = (it + t) % 8
                if t % 2 == 0 and it % 6 == 0:
                    da.da_spmm_prepare(a.m, a.k, a.nnz, job["rp"], job["ci"], stream=job["stream"])
                if t % 2 == 0 and it % 6 == 5:
                    da.da_spmm_release(job["rp"])
                da.da_spmm(a.m, a.k, N, job["rp"], job["ci"], job["va"], job["B"], job["C"], algo,
                           stream=job["stream"])
                job["stream"].synchronize()
                c = job["C"].cpu().numpy()
                job["worst"] = max(job["worst"], orc.tolerance_ratio(c, job["ref"], job["s_abs"]))
        except Exception as e:                      # reported by the main thread
            job["error"] = repr(e)

    threads = [threading.Thread(target=work, args=(t, job)) for t, job in enumerate(jobs)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    for job in jobs:
        da.da_spmm_release(job["rp"])
        assert job["error"] is None, job["error"]
        assert job["worst"] <= 1.0
