"""da_csr_transpose_noalloc (the entry point that allocates nothing: static device scratch) against
da_csr_transpose with a caller workspace, bit for bit, on two calls in a row that share the
library's scratch array, the second on a smaller matrix; and against the oracle's transpose.  This
file is collected last on purpose: it must pass alone in a fresh process and after all other tests."""
import numpy as np
import pytest
import torch

from oracle import reference as orc
from paper_2202_08556_amd import generators as gen

pytestmark = pytest.mark.gpu


def transpose_both_ways(a):
    """(result through the workspace entry point, result through the no-allocation entry point)."""
    from paper_2202_08556_amd import binding as da
    dev = torch.device("cuda:0")
    rp, ci, va = (torch.from_numpy(np.ascontiguousarray(x)).to(dev) for x in (a.rowptr, a.colind, a.vals))
    nnz = int(a.colind.size)

    def outputs():
        return (torch.full((a.k + 1,), -7, dtype=torch.int32, device=dev),
                torch.full((nnz,), -7, dtype=torch.int32, device=dev),
                torch.full((nnz,), float("nan"), dtype=torch.float32, device=dev))

    nbytes = da.da_csr_transpose_workspace(a.m, a.k, nnz)
    assert nbytes <= da.DA_NOALLOC_SCRATCH_BYTES
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    ref = outputs()
    da.da_csr_transpose(a.m, a.k, nnz, rp, ci, va, *ref, ws, nbytes)
    got = outputs()
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    da.da_csr_transpose_noalloc(a.m, a.k, nnz, rp, ci, va, *got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return [x.cpu().numpy() for x in ref], [x.cpu().numpy() for x in got]


def test_noalloc_transpose_twice_second_call_smaller():
    big = gen.powerlaw_csr(m=16384, seed=2002)                      # ~0.8 M entries, three radix passes
    small = gen.uniform_csr(m=1237, k=911, mean_len=11, seed=7)      # one pass, a fraction of the scratch
    assert small.nnz < big.nnz
    for a in (big, small):
        print(f"noalloc transpose {a.name} m={a.m} k={a.k} nnz={a.nnz}", flush=True)
        ref, got = transpose_both_ways(a)
        for r, g in zip(ref, got):
            assert np.array_equal(r.view(np.uint32), g.view(np.uint32))
        want = orc.csr_transpose(a.rowptr, a.colind, a.vals, a.k)
        assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
        assert np.array_equal(got[2].view(np.uint32), want[2].view(np.uint32))


def test_noalloc_transpose_rejects_what_does_not_fit_and_handles_empty():
    from paper_2202_08556_amd import binding as da
    dev = torch.device("cuda:0")
    # size check comes before any device access: dummy one-element buffers are never touched
    one_i = torch.zeros(1, dtype=torch.int32, device=dev)
    one_f = torch.zeros(1, dtype=torch.float32, device=dev)
    nnz = 3_000_000
    assert da.da_csr_transpose_workspace(1000, 1000, nnz) > da.DA_NOALLOC_SCRATCH_BYTES
    st = da.da_csr_transpose_noalloc_status(1000, 1000, nnz, one_i, one_i, one_f, one_i, one_i, one_f)
    assert st == da.DA_ERR_UNSUPPORTED
    assert "32 MiB" in da.da_spmm_last_error()
    assert da.da_csr_transpose_noalloc_status(-1, 5, 0, one_i, one_i, one_f, one_i, one_i, one_f) == da.DA_ERR_INVALID_ARG
    # no stored entries: row pointers of the transpose are all zero
    t_rp = torch.full((10,), -7, dtype=torch.int32, device=dev)
    rp = torch.zeros(6, dtype=torch.int32, device=dev)
    da.da_csr_transpose_noalloc(5, 9, 0, rp, None, None, t_rp, None, None)
    torch.cuda.synchronize()
    assert np.array_equal(t_rp.cpu().numpy(), np.zeros(10, dtype=np.int32))
