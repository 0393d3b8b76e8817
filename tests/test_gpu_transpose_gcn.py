"""da_csr_transpose against the oracle's transpose (bit for bit: index work and copied values), and
the graph-convolution layer (aggregation A.X forward, A^T.dY backward, Sec. 6) against the fp64
oracle within the SpMM tolerance |C - C_ref| <= 1e-5 * (|A|.|B|)_ij + 1e-6."""
import numpy as np
import pytest
import torch

from oracle import reference as orc
from paper_2202_08556_amd import generators as gen

pytestmark = pytest.mark.gpu


def heavy_column():
    """70001 rows with one entry each, all but a few in column 3: one digit takes whole blocks."""
    m, k = 70001, 50
    colind = np.full(m, 3, dtype=np.int32)
    colind[::1000] = 49
    colind[5] = 0
    vals = np.arange(m, dtype=np.float32)
    return gen.CSR(m=m, k=k, rowptr=np.arange(m + 1, dtype=np.int32), colind=colind, vals=vals, seed=0, name="heavy_column")


def duplicates_unsorted():
    """Rows whose columns are not sorted and repeat: stored order must survive among equal (row, column)."""
    rng = np.random.default_rng(77)
    m, k = 300, 40
    lens = rng.integers(0, 30, size=m)
    rowptr = np.zeros(m + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum(lens)
    colind = rng.integers(0, k, size=int(rowptr[-1])).astype(np.int32)
    vals = rng.standard_normal(int(rowptr[-1])).astype(np.float32)
    return gen.CSR(m=m, k=k, rowptr=rowptr, colind=colind, vals=vals, seed=77, name="duplicates_unsorted")


def transpose_cases():
    yield gen.fig6a_csr()
    yield gen.uniform_csr(m=37, k=53, mean_len=5, seed=31)                      # one pass (k <= 1024)
    yield gen.uniform_csr(m=1237, k=911, mean_len=11, seed=7)
    yield gen.lognormal_csr(3000, 12.0, 3.0, seed=35, name="lognormal")        # two passes
    yield gen.powerlaw_csr(m=8192, seed=2001)                                   # hot columns, several blocks
    yield gen.skewed_csr(m=16384, heavy_lo=3000, heavy_hi=9000, seed=4001)
    yield gen.stencil27_csr(12, 13, 14, seed=3001)
    yield gen.uniform_csr(m=5000, k=1200000, mean_len=20, seed=51)              # three passes, wide and mostly empty A^T
    yield gen.uniform_csr(m=100000, k=7, mean_len=3, seed=52)                   # tall: 7 long rows in A^T
    yield heavy_column()
    yield duplicates_unsorted()
    yield gen.CSR(m=5, k=9, rowptr=np.zeros(6, dtype=np.int32), colind=np.zeros(0, np.int32),
                  vals=np.zeros(0, np.float32), seed=0, name="no_entries")


def device_transpose(a, sentinel=True):
    from paper_2202_08556_amd import binding as da
    dev = torch.device("cuda:0")
    rp, ci, va = (torch.from_numpy(np.ascontiguousarray(x)).to(dev) for x in (a.rowptr, a.colind, a.vals))
    nnz = int(a.colind.size)
    t_rp = torch.full((a.k + 1,), -7, dtype=torch.int32, device=dev)
    t_ci = torch.full((nnz,), -7, dtype=torch.int32, device=dev)
    t_va = torch.full((nnz,), float("nan"), dtype=torch.float32, device=dev)
    nbytes = da.da_csr_transpose_workspace(a.m, a.k, nnz)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    da.da_csr_transpose(a.m, a.k, nnz, rp, ci, va, t_rp, t_ci, t_va, ws, nbytes)
    torch.cuda.synchronize()
    return t_rp.cpu().numpy(), t_ci.cpu().numpy(), t_va.cpu().numpy()


@pytest.mark.parametrize("a", list(transpose_cases()), ids=lambda a: a.name)
def test_transpose_matches_oracle_bit_for_bit(a):
    print(f"transpose case {a.name} m={a.m} k={a.k} nnz={a.colind.size}", flush=True)
    ref = orc.csr_transpose(a.rowptr, a.colind, a.vals, a.k)
    got = device_transpose(a)
    assert np.array_equal(got[0], ref[0])
    assert np.array_equal(got[1], ref[1])
    assert np.array_equal(got[2].view(np.uint32), ref[2].view(np.uint32))


def test_transpose_is_deterministic_and_its_own_inverse():
    a = gen.powerlaw_csr(m=8192, seed=2001)
    t1 = device_transpose(a)
    t2 = device_transpose(a)
    assert all(np.array_equal(x, y) for x, y in zip(t1, t2))
    back = device_transpose(gen.CSR(m=a.k, k=a.m, rowptr=t1[0], colind=t1[1], vals=t1[2], seed=0, name="t"))
    assert np.array_equal(back[0], a.rowptr) and np.array_equal(back[1], a.colind) and np.array_equal(back[2], a.vals)


def test_transpose_argument_errors():
    from paper_2202_08556_amd import binding as da
    dev = torch.device("cuda:0")
    a = gen.uniform_csr(m=37, k=53, mean_len=5, seed=31)
    nnz = int(a.colind.size)
    rp, ci, va = (torch.from_numpy(x).to(dev) for x in (a.rowptr, a.colind, a.vals))
    t_rp = torch.zeros(a.k + 1, dtype=torch.int32, device=dev)
    t_ci = torch.zeros(nnz, dtype=torch.int32, device=dev)
    t_va = torch.zeros(nnz, dtype=torch.float32, device=dev)
    nbytes = da.da_csr_transpose_workspace(a.m, a.k, nnz)
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
    bad = da.DA_ERR_INVALID_ARG
    assert da.da_csr_transpose_status(a.m, a.k, nnz, rp, ci, va, t_rp, t_ci, t_va, ws, nbytes - 1) == bad
    assert "workspace" in da.da_spmm_last_error()
    assert da.da_csr_transpose_status(a.m, a.k, nnz, rp, ci, va, t_rp, t_ci, t_va, None, 0) == bad
    assert da.da_csr_transpose_status(a.m, a.k, nnz, rp, ci, va, t_rp, t_ci, t_va, ws.data_ptr() + 4, nbytes) == bad
    assert da.da_csr_transpose_status(-1, a.k, nnz, rp, ci, va, t_rp, t_ci, t_va, ws, nbytes) == bad
    assert da.da_csr_transpose_status(a.m, a.k, nnz, rp, None, va, t_rp, t_ci, t_va, ws, nbytes) == bad
    assert da.da_csr_transpose_status(a.m, a.k, 1 << 31, rp, ci, va, t_rp, t_ci, t_va, ws, nbytes) == bad
    assert da.da_csr_transpose_status(a.m, a.k, nnz, rp, ci, va, t_rp, t_ci, t_va, ws, nbytes) == da.DA_OK
    torch.cuda.synchronize()


GRAPHS = [("powerlaw", lambda: gen.powerlaw_csr(m=4096, seed=2101), [16, 64]),
          ("rect_lognormal", lambda: gen.lognormal_csr(3000, 12.0, 3.0, seed=35, name="ln"), [32]),
          ("rect_uniform", lambda: gen.uniform_csr(m=1237, k=911, mean_len=11, seed=7), [20, 256])]


@pytest.mark.parametrize("name,make,Ns", GRAPHS, ids=[g[0] for g in GRAPHS])
def test_aggregate_forward_and_backward_match_oracle(name, make, Ns):
    from paper_2202_08556_amd import gcn
    a = make()
    graph = gcn.SparseGraph.from_numpy(a)
    for N in Ns:
        print(f"aggregate case {name} N={N}", flush=True)
        X = gen.dense(a.k, N, "normal", seed=a.seed + N)
        G = gen.dense(a.m, N, "uniform", seed=a.seed + N + 1)
        Xd = torch.from_numpy(X).cuda().requires_grad_(True)
        Y = gcn.aggregate(graph, Xd)
        Y.backward(torch.from_numpy(G).cuda())
        torch.cuda.synchronize()
        c_ref, s_abs = orc.spmm(a.rowptr, a.colind, a.vals, X)
        assert orc.tolerance_ratio(Y.detach().cpu().numpy(), c_ref, s_abs) <= 1.0
        d_ref, sd_abs = orc.spmm_transposed(a.rowptr, a.colind, a.vals, G, a.k)
        assert orc.tolerance_ratio(Xd.grad.cpu().numpy(), d_ref, sd_abs) <= 1.0


def test_backward_exact_on_integer_inputs():
    from paper_2202_08556_amd import gcn
    a = gen.integer_twin(gen.powerlaw_csr(m=4096, seed=2102))
    N = 32
    G = gen.dense_int(a.m, N, seed=9)
    graph = gcn.SparseGraph.from_numpy(a)
    Xd = torch.zeros((a.k, N), device="cuda:0", requires_grad=True)
    gcn.aggregate(graph, Xd).backward(torch.from_numpy(G).cuda())
    torch.cuda.synchronize()
    d_ref, _ = orc.spmm_transposed(a.rowptr, a.colind, a.vals, G, a.k)
    assert orc.bit_mismatches(Xd.grad.cpu().numpy(), d_ref) == 0


def test_graph_conv_layer_matches_fp64_layer():
    """Whole layer relu(A.(X.W)+b), forward and all three gradients.  The dense products run in the
    fp32 GEMM library, so the bound is a relative one on the size of each result."""
    from paper_2202_08556_amd import gcn
    a = gen.powerlaw_csr(m=2048, seed=2103)
    fin, fout = 48, 32
    rng = np.random.default_rng(5)
    X = rng.standard_normal((a.m, fin)).astype(np.float32)
    d_out = rng.standard_normal((a.m, fout)).astype(np.float32)
    torch.manual_seed(3)
    layer = gcn.GraphConv(fin, fout).cuda()
    with torch.no_grad():
        layer.bias.uniform_(-0.1, 0.1)
    W = layer.weight.detach().cpu().numpy()
    b = layer.bias.detach().cpu().numpy()
    ref_out, Z = orc.gcn_layer(a.rowptr, a.colind, a.vals, X, W, b)
    # a unit whose pre-activation is within rounding of zero may fall on either side of the relu in
    # fp32: give those units no incoming gradient, so that the comparison does not hinge on them
    d_out[np.abs(Z) <= 1e-4] = 0.0
    dX, dW, db = orc.gcn_layer_backward(a.rowptr, a.colind, a.vals, X, W, Z, d_out)
    graph = gcn.SparseGraph.from_numpy(a)
    Xd = torch.from_numpy(X).cuda().requires_grad_(True)
    out = layer(graph, Xd)
    out.backward(torch.from_numpy(d_out).cuda())
    torch.cuda.synchronize()
    got = out.detach().cpu().numpy()
    assert np.max(np.abs(got - ref_out)) <= 2e-5 * np.max(np.abs(ref_out)) + 1e-6
    for g, r in ((Xd.grad, dX), (layer.weight.grad, dW), (layer.bias.grad, db)):
        assert np.max(np.abs(g.cpu().numpy() - r)) <= 5e-5 * np.max(np.abs(r)) + 1e-6


# ---- EB chunk schedule (da_eb_schedule, da_spmm_prepare) -------------------------------------
def schedule_cases():
    yield gen.skewed_csr(m=16384, heavy_lo=3000, heavy_hi=9000, seed=4001), (64, 256, 512)
    yield gen.powerlaw_csr(m=8192, seed=2001), (64, 128)
    yield gen.uniform_csr(m=5000, k=1200000, mean_len=20, seed=51), (1, 64)
    yield gen.uniform_csr(m=37, k=53, mean_len=5, seed=31), (7, 512)


def check_schedule_properties(a, unit, order, first_segment):
    """What include/da_spmm.h promises of da_eb_schedule's output, checked from the matrix itself.
    The order is the library's own heuristic (any permutation of the chunks gives the same product,
    which the parity tests check), so there is no oracle for it: the stated properties are verified
    one by one from per-entry row numbers and the column indices the chunks actually hold."""
    nnz = int(a.colind.size)
    nunits = -(-nnz // unit)
    order = np.asarray(order, dtype=np.int64)
    assert order.shape == (nunits,)
    assert np.array_equal(np.sort(order), np.arange(nunits))                 # a permutation of the chunks
    row_of = np.repeat(np.arange(a.m), np.diff(a.rowptr))
    first = np.arange(nunits, dtype=np.int64) * unit
    last = np.minimum(first + unit, nnz) - 1
    several = row_of[first] != row_of[last]                                   # the chunk touches several rows
    assert first_segment == int(several.sum())
    assert several[order[:first_segment]].all() and not several[order[first_segment:]].any()
    col = a.colind.astype(np.int64)
    for seg, seen in ((order[:first_segment], col[first]),                    # swept by first column
                      (order[first_segment:], (col[first] + col[last]) // 2)):  # swept by the middle of the range
        key = seen[seg]
        assert np.all(np.diff(key) >= 0)                                      # a sweep from low to high columns
        tie = np.diff(key) == 0
        assert np.all(np.diff(seg)[tie] > 0)                                  # equal keys: ascending chunk number


@pytest.mark.parametrize("a,units", list(schedule_cases()), ids=lambda x: getattr(x, "name", None))
def test_eb_schedule_has_the_promised_properties(a, units):
    from paper_2202_08556_amd import binding as da
    dev = torch.device("cuda:0")
    ci = torch.from_numpy(a.colind).to(dev)
    rp = torch.from_numpy(a.rowptr).to(dev)
    nnz = int(a.colind.size)
    for unit in units:
        print(f"schedule case {a.name} unit={unit}", flush=True)
        nunits = -(-nnz // unit)
        order = torch.full((nunits,), -3, dtype=torch.int32, device=dev)
        seg = torch.full((1,), -3, dtype=torch.int32, device=dev)
        nbytes = da.da_eb_schedule_workspace(a.k, nnz, unit)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        da.da_eb_schedule(a.m, a.k, nnz, rp, ci, unit, order, seg, ws, nbytes)
        torch.cuda.synchronize()
        first_order = order.cpu().numpy().copy()
        check_schedule_properties(a, unit, first_order, int(seg.item()))
        order.fill_(-3)
        da.da_eb_schedule(a.m, a.k, nnz, rp, ci, unit, order, None, ws, nbytes)      # the count is optional
        torch.cuda.synchronize()
        assert np.array_equal(order.cpu().numpy(), first_order)                     # and the result deterministic
    assert da.da_eb_schedule_status(a.m, a.k, nnz, rp, ci, 64, order, None, ws, 8) == da.DA_ERR_INVALID_ARG
    assert da.da_eb_schedule_status(a.m, a.k, nnz, rp, ci, 0, order, None, ws, nbytes) == da.DA_ERR_INVALID_ARG
    assert da.da_eb_schedule_status(a.m, a.k, nnz, None, ci, 64, order, None, ws, nbytes) == da.DA_ERR_INVALID_ARG


def rows_around_the_chunk_size(seed=71):
    """Row lengths at and around the EB+SR chunk sizes (128, 256), rows that begin or end exactly
    on chunk boundaries, runs of rows without entries and single-entry rows in between: the shapes
    the rule "rows of at most a chunk are never split" has to get right."""
    rng = np.random.default_rng(seed)
    menu = np.array([0, 0, 1, 2, 127, 128, 129, 255, 256, 257, 300, 511, 512, 513, 1024, 33, 64])
    lens = rng.choice(menu, size=1500)
    lens[:8] = [256, 256, 128, 128, 0, 256, 255, 1]                 # boundaries that fall on row starts
    lens[100:140] = 0                                               # a run of rows without entries
    k = 6000
    rowptr, colind = gen.csr_from_lens(rng, lens, k)
    vals = rng.uniform(-1, 1, size=colind.size).astype(np.float32)
    return gen.CSR(m=len(lens), k=k, rowptr=rowptr.astype(np.int32), colind=colind.astype(np.int32), vals=vals,
                   seed=seed, name="rows_around_chunk")


PREPARED = [("skewed", lambda: gen.skewed_csr(m=16384, heavy_lo=3000, heavy_hi=9000, seed=4001), [8, 64]),
            ("powerlaw", lambda: gen.powerlaw_csr(m=8192, seed=2001), [32, 128]),
            ("one_long_row", lambda: gen.skewed_csr(m=64, k=40000, heavy_frac=0.02, heavy_lo=30000, heavy_hi=30000,
                                                    light_mean=0.5, seed=9), [8]),
            # several column tiles (520 = 2*256 + 8), a ragged N without 16-byte accesses, and enough
            # chunks for several rounds of XCD stripes at the smallest chunk size
            ("wide_and_ragged_N", lambda: gen.skewed_csr(m=20000, k=15000, heavy_frac=0.01, heavy_lo=4000,
                                                         heavy_hi=9000, seed=12), [520, 13]),
            ("few_entries", lambda: gen.uniform_csr(m=9, k=11, mean_len=3, seed=5), [4]),
            # lane groups of 32 / 16 (rows of at most a chunk stay whole) and of 8 (they are split)
            ("rows_around_chunk", rows_around_the_chunk_size, [128, 64, 32]),
            ("hypersparse", lambda: gen.hypersparse_csr(200000, 25000, 0.01, 100.0, seed=73), [128])]


@pytest.mark.parametrize("name,make,Ns", PREPARED, ids=[p[0] for p in PREPARED])
def test_prepared_matrix_all_algorithms_match_oracle(name, make, Ns):
    """After da_spmm_prepare the EB ids run with the column-sweep chunk order; every id must still
    match the oracle, also on the integer twin bit for bit, and also after the plan went stale."""
    from paper_2202_08556_amd import binding as da
    from tests.gpu_util import DeviceProblem
    a = make()
    try:
        for N in Ns:
            B = gen.dense(a.k, N, "uniform", seed=a.seed + N)
            c_ref, s_abs = orc.spmm(a.rowptr, a.colind, a.vals, B)
            prob = DeviceProblem(a, B)
            da.da_spmm_prepare(a.m, a.k, a.nnz, prob.rowptr, prob.colind)
            for algo in range(8):
                print(f"prepared case {name} N={N} algo={algo}", flush=True)
                assert orc.tolerance_ratio(prob.run(algo), c_ref, s_abs) <= 1.0, (name, N, algo)
            # stale plan: other contents (fewer entries) in the same buffers
            half = gen.CSR(m=a.m, k=a.k, rowptr=np.minimum(a.rowptr, a.rowptr[a.m // 2]).astype(np.int32),
                           colind=a.colind, vals=a.vals, seed=a.seed, name="half")
            prob.rowptr.copy_(torch.from_numpy(half.rowptr))
            c_half, s_half = orc.spmm(half.rowptr, half.colind[:half.rowptr[-1]], half.vals[:half.rowptr[-1]], B)
            for algo in (4, 5, 6, 7):
                print(f"stale plan case {name} N={N} algo={algo}", flush=True)
                assert orc.tolerance_ratio(prob.run(algo), c_half, s_half) <= 1.0, (name, N, algo)
            da.da_spmm_release(prob.rowptr)
        ai = gen.integer_twin(a)
        Bi = gen.dense_int(a.k, Ns[0], seed=3)
        c_int, _ = orc.spmm(ai.rowptr, ai.colind, ai.vals, Bi, want_abs=False)
        prob = DeviceProblem(ai, Bi)
        da.da_spmm_prepare(ai.m, ai.k, ai.nnz, prob.rowptr, prob.colind)
        for algo in (4, 5, 6, 7):
            assert orc.bit_mismatches(prob.run(algo), c_int) == 0, (name, algo)
    finally:
        da.da_spmm_release()


def test_prepared_buffers_reused_for_another_matrix_of_equal_nnz():
    """The plan is keyed by (rowptr address, colind address, m) and guarded by nnz only: when the
    same buffers later hold another matrix with the same number of rows and stored entries the old
    chunk order is applied to it.  Any order of the chunks is a valid one, and the rows that need
    zeroing or atomics are decided from the row pointers at run time, so the product must still be
    that of the new matrix."""
    from paper_2202_08556_amd import binding as da
    from tests.gpu_util import DeviceProblem
    a1 = gen.skewed_csr(m=16384, heavy_lo=3000, heavy_hi=9000, seed=4001)
    rng = np.random.default_rng(99)
    lens = np.diff(a1.rowptr)[::-1].copy()                       # long rows move elsewhere
    rowptr = np.zeros(a1.m + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum(lens)
    colind = np.concatenate([np.sort(rng.integers(0, a1.k, size=n)) for n in lens]).astype(np.int32)
    a2 = gen.CSR(m=a1.m, k=a1.k, rowptr=rowptr, colind=colind,
                 vals=rng.uniform(-1, 1, size=colind.size).astype(np.float32), seed=99, name="reused")
    assert a2.nnz == a1.nnz and not np.array_equal(a1.rowptr, a2.rowptr)
    N = 64
    B = gen.dense(a1.k, N, "uniform", seed=5)
    prob = DeviceProblem(a1, B)
    try:
        da.da_spmm_prepare(a1.m, a1.k, a1.nnz, prob.rowptr, prob.colind)
        prob.a = a2
        prob.rowptr.copy_(torch.from_numpy(a2.rowptr))
        prob.colind.copy_(torch.from_numpy(a2.colind))
        prob.vals.copy_(torch.from_numpy(a2.vals))
        c_ref, s_abs = orc.spmm(a2.rowptr, a2.colind, a2.vals, B)
        for algo in range(8):
            print(f"reused buffers algo={algo}", flush=True)
            assert orc.tolerance_ratio(prob.run(algo), c_ref, s_abs) <= 1.0, algo
        ai = gen.integer_twin(a2)
        Bi = gen.dense_int(a2.k, N, seed=6)
        prob.vals.copy_(torch.from_numpy(ai.vals))
        prob.B.copy_(torch.from_numpy(Bi))
        c_int, _ = orc.spmm(ai.rowptr, ai.colind, ai.vals, Bi, want_abs=False)
        for algo in (4, 5, 6, 7):
            assert orc.bit_mismatches(prob.run(algo), c_int) == 0, algo
    finally:
        da.da_spmm_release()


def test_prepare_edge_cases_and_release():
    from paper_2202_08556_amd import binding as da
    dev = torch.device("cuda:0")
    a = gen.uniform_csr(m=300, k=200, mean_len=6, seed=61)
    rp, ci = torch.from_numpy(a.rowptr).to(dev), torch.from_numpy(a.colind).to(dev)
    da.da_spmm_prepare(0, 5, 0, None, None)                        # nothing to prepare
    da.da_spmm_prepare(a.m, a.k, 0, rp, ci)
    with pytest.raises(da.DaSpmmError):
        da.da_spmm_prepare(a.m, a.k, a.nnz, None, ci)
    with pytest.raises(da.DaSpmmError):
        da.da_spmm_prepare(-1, a.k, a.nnz, rp, ci)
    for _ in range(20):                                            # more plans than the table holds: old ones are freed
        r2 = rp.clone()
        da.da_spmm_prepare(a.m, a.k, a.nnz, r2, ci)
    da.da_spmm_prepare(a.m, a.k, a.nnz, rp, ci)
    da.da_spmm_prepare(a.m, a.k, a.nnz, rp, ci)                    # preparing twice replaces the plan
    da.da_spmm_release(rp)
    da.da_spmm_release(rp)                                         # releasing an unknown matrix is not an error
    da.da_spmm_release()
