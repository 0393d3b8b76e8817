"""The largest index range the ABI allows: a matrix with 1.6 G stored entries (int32 row pointers up
to 1.6e9, close to the 2^31 limit), built on the device from closed-form index patterns.  Every
algorithm id, unprepared and prepared, is compared bit for bit (integer-valued data) with the
oracle on a sample of rows: the oracle receives a small CSR matrix that holds exactly those rows."""
import numpy as np
import pytest
import torch

from oracle import reference as orc

pytestmark = pytest.mark.gpu

M, K, L, N = 1 << 22, 1 << 22, 384, 8            # 4 Mi rows of 384 entries = 1 610 612 736 entries


def build_on_device(dev):
    rowptr = (torch.arange(M + 1, dtype=torch.int64, device=dev) * L).to(torch.int32)
    colind = torch.empty(M * L, dtype=torch.int32, device=dev)
    vals = torch.empty(M * L, dtype=torch.float32, device=dev)
    t = torch.arange(L, dtype=torch.int64, device=dev)
    step = 1 << 16                                 # rows per slab, keeps temporaries at a few hundred MB
    for r0 in range(0, M, step):
        rows = torch.arange(r0, min(M, r0 + step), dtype=torch.int64, device=dev)[:, None]
        col = (rows * 131 + t[None, :] * 10007 + (rows >> 7)) % K
        val = ((rows * 7 + t[None, :] * 3) % 6) - 3          # -3..2
        val = torch.where(val >= 0, val + 1, val)             # {-3,-2,-1,1,2,3}
        colind[r0 * L:(r0 + rows.shape[0]) * L] = col.reshape(-1).to(torch.int32)
        vals[r0 * L:(r0 + rows.shape[0]) * L] = val.reshape(-1).to(torch.float32)
    return rowptr, colind, vals


def test_largest_index_range_bit_exact():
    from paper_2202_08556_amd import binding as da
    dev = torch.device("cuda:0")
    print("building 1.6 G-entry matrix on the device", flush=True)
    rowptr, colind, vals = build_on_device(dev)
    nnz = M * L
    assert int(rowptr[-1].item()) == nnz and nnz >= (3 << 29)
    g = torch.Generator(device="cpu"); g.manual_seed(5)
    B_host = torch.randint(-4, 5, (K, N), generator=g, dtype=torch.int32).to(torch.float32)
    B = B_host.to(dev)
    C = torch.empty((M, N), dtype=torch.float32, device=dev)
    rng = np.random.default_rng(6)
    rows = np.unique(np.concatenate([rng.integers(0, M, size=3000), [0, 1, M - 2, M - 1]])).astype(np.int64)
    # the sampled rows as a CSR matrix of their own, for the oracle
    idx = (torch.from_numpy(rows).to(dev)[:, None] * L + torch.arange(L, device=dev)[None, :]).reshape(-1)
    sub_colind = colind[idx].cpu().numpy()
    sub_vals = vals[idx].cpu().numpy()
    sub_rowptr = (np.arange(rows.size + 1, dtype=np.int64) * L).astype(np.int32)
    c_ref, _ = orc.spmm(sub_rowptr, sub_colind, sub_vals, B_host.numpy(), want_abs=False)
    da.da_csr_validate(M, K, nnz, rowptr, colind)
    feats = da.da_spmm_features(M, N, rowptr)
    assert feats["nnz"] == nnz and feats["row_nnz_max"] == L and feats["row_nnz_std"] == 0.0
    rows_dev = torch.from_numpy(rows).to(dev)
    for prepared in (False, True):
        if prepared:
            print("da_spmm_prepare at 1.6 G entries", flush=True)
            da.da_spmm_prepare(M, K, nnz, rowptr, colind)
        for algo in range(8):
            print(f"max-size case prepared={prepared} algo={algo}", flush=True)
            C.fill_(float("nan"))
            da.da_spmm(M, K, N, rowptr, colind, vals, B, C, algo)
            torch.cuda.synchronize()
            assert orc.bit_mismatches(C[rows_dev].cpu().numpy(), c_ref) == 0, (prepared, algo)
            assert bool(torch.isfinite(C).all())
    da.da_spmm_release(rowptr)


def test_operands_beyond_4_gib_take_the_wide_kernels():
    """B and C of 8 GiB each (2^21 x 1024 floats): element offsets exceed 32 bits, so the library must
    use its 64-bit gather addressing by itself.  Integer data, bit-exact on sampled rows; the oracle
    gets the sampled rows with their columns renumbered onto a compact copy of the B rows they use."""
    from paper_2202_08556_amd import binding as da
    dev = torch.device("cuda:0")
    m = k = 1 << 21
    N, per_row = 1024, 3
    rows_all = torch.arange(m, dtype=torch.int64, device=dev)
    rowptr = (torch.arange(m + 1, dtype=torch.int64, device=dev) * per_row).to(torch.int32)
    t = torch.arange(per_row, dtype=torch.int64, device=dev)
    colind = ((rows_all[:, None] * 977 + t[None, :] * 699053 + 5) % k).reshape(-1).to(torch.int32)
    vals = (((rows_all[:, None] + t[None, :]) % 3) + 1).reshape(-1).to(torch.float32)
    nnz = m * per_row

    def b_values(r, n):                                   # closed form, same on host and device
        return ((r * 31 + n * 17) % 9) - 4

    B = torch.empty((k, N), dtype=torch.float32, device=dev)
    ncol = torch.arange(N, dtype=torch.int64, device=dev)
    for r0 in range(0, k, 1 << 17):
        r = torch.arange(r0, min(k, r0 + (1 << 17)), dtype=torch.int64, device=dev)
        B[r0:r0 + r.shape[0]] = b_values(r[:, None], ncol[None, :]).to(torch.float32)
    C = torch.empty((m, N), dtype=torch.float32, device=dev)
    assert B.numel() * 4 > (1 << 32)
    rng = np.random.default_rng(8)
    rows = np.unique(np.concatenate([rng.integers(0, m, size=1500), [0, m - 1]])).astype(np.int64)
    idx = (torch.from_numpy(rows).to(dev)[:, None] * per_row + t[None, :]).reshape(-1)
    sub_cols = colind[idx].cpu().numpy().astype(np.int64)
    used, compact = np.unique(sub_cols, return_inverse=True)
    B_small = b_values(used[:, None], np.arange(N, dtype=np.int64)[None, :]).astype(np.float32)
    sub_rowptr = (np.arange(rows.size + 1, dtype=np.int64) * per_row).astype(np.int32)
    c_ref, _ = orc.spmm(sub_rowptr, compact.astype(np.int32), vals[idx].cpu().numpy(), B_small, want_abs=False)
    da.da_spmm_features(m, N, rowptr)
    rows_dev = torch.from_numpy(rows).to(dev)
    for algo in range(8):
        print(f"beyond-4-GiB case algo={algo}", flush=True)
        C.fill_(float("nan"))
        da.da_spmm(m, k, N, rowptr, colind, vals, B, C, algo)
        torch.cuda.synchronize()
        assert orc.bit_mismatches(C[rows_dev].cpu().numpy(), c_ref) == 0, algo
        assert bool(torch.isfinite(C[-4096:]).all()) and bool(torch.isfinite(C[:4096]).all())
