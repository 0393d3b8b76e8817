"""Controlled experiments of the paper's Sec. 6.3 on seeded R-MAT matrices (one GPU).

    python -m paper_2202_08556_amd.controlled > results/controlled.txt

  RB-EB  three matrices of identical size and sparsity whose rows are more and more dispersed
         (R-MAT quadrant probabilities from uniform to strongly skewed): best RB id against best EB id
  RM-CM  one matrix, growing dense width N: best RM id against best CM id
  SR-PR  one distribution, growing size: best SR id against best PR id

The paper prints neither its R-MAT parameters nor its sizes; the ones used here are listed in the
output.  Times are HIP-event times per call, rotating over 3 copies of B and C.
"""
from __future__ import annotations

import sys

import numpy as np
import torch

from . import binding as da
from . import generators as gen
from .sweep import COPIES, time_algo

RB, EB = (0, 1, 2, 3), (4, 5, 6, 7)
RM, CM = (0, 1, 4, 5), (2, 3, 6, 7)
SR, PR = (0, 2, 4, 6), (1, 3, 5, 7)


def time_all(a, N, col_major=False):
    """Times of the 8 ids; with col_major both B and C are stored column-major (da_spmm_ex)."""
    dev = torch.device("cuda:0")
    rp, ci, va = (torch.from_numpy(x).to(dev) for x in (a.rowptr, a.colind, a.vals))
    da.da_spmm_features(a.m, N, rp)
    da.da_spmm_prepare(a.m, a.k, a.nnz, rp, ci)                 # EB chunk order, as a user would
    g = torch.Generator(device=dev)
    g.manual_seed(a.seed * 1000 + N)
    Bs = [torch.empty((a.k, N), device=dev).uniform_(-1.0, 1.0, generator=g) for _ in range(COPIES)]
    Cs = [torch.empty((a.m, N), device=dev) for _ in range(COPIES)]
    lay = da.DA_COL_MAJOR if col_major else da.DA_ROW_MAJOR     # the buffers are just reinterpreted
    runs = [da.PreparedSpmm(a.m, a.k, N, rp, ci, va, Bs[i], Cs[i], layout_b=lay, layout_c=lay) for i in range(COPIES)]
    times = []
    for algo in range(da.DA_NUM_ALGOS):
        t, _ = time_algo(lambda i, algo=algo: runs[i % COPIES](algo))
        times.append(t)
    da.da_spmm_release(rp)
    return np.array(times)


def best(times, ids):
    i = min(ids, key=lambda a: times[a])
    return times[i], da.ALGO_NAMES[i]


def line(label, times, left, right, lname, rname):
    tl, nl = best(times, left)
    tr, nr = best(times, right)
    print(f"{label:58s} {lname} {tl:9.1f} us ({nl})   {rname} {tr:9.1f} us ({nr})   {lname}/{rname} time ratio {tl / tr:6.2f}",
          flush=True)


def main():
    from .profile_summary import source_hash
    print("Controlled experiments of the paper's Sec. 6.3 (Fig. 9) on seeded R-MAT matrices, one MI355X, fp32.")
    print("command (repository root, after __graft_entry__.build()):  python -m paper_2202_08556_amd.controlled")
    print(f"SOURCE_SHA256 = {source_hash()}")
    print("HIP-event time per call (EB ids include the zero pre-pass), best id of each side of the axis; B and C rotate "
          "over 3 copies.")
    print("Matrices are prepared with da_spmm_prepare (EB chunk order) before timing.\n")
    print("RB-EB: R-MAT scale 17 (131072 rows), 16 entries per row on average, N = 32")
    for i, (a, b, c) in enumerate(((0.25, 0.25, 0.25), (0.45, 0.22, 0.22), (0.57, 0.19, 0.19))):
        m = gen.rmat_csr(17, 16.0, a, b, c, seed=8200 + i)
        lens = m.row_lengths()
        line(f"  (a,b,c)=({a},{b},{c}) std of row length {lens.std():7.1f} max {lens.max():6d}",
             time_all(m, 32), RB, EB, "RB", "EB")
    print("RM-CM: R-MAT scale 17, (a,b,c)=(0.45,0.22,0.22), 16 entries per row")
    m = gen.rmat_csr(17, 16.0, 0.45, 0.22, 0.22, seed=8210)
    for N in (2, 4, 8, 32, 128):
        line(f"  N = {N}", time_all(m, N), RM, CM, "RM", "CM")
    print("stored layouts (Sec. 3.3 literally): same matrix, best of the 8 ids with B and C row-major against column-major")
    for N in (2, 4, 8, 32, 128):
        tr, tc = time_all(m, N), time_all(m, N, col_major=True)
        ir, ic = int(np.argmin(tr)), int(np.argmin(tc))
        print(f"  N = {N:3d}   row-major {tr[ir]:9.1f} us ({da.ALGO_NAMES[ir]})   column-major {tc[ic]:9.1f} us ({da.ALGO_NAMES[ic]})"
              f"   row/column time ratio {tr[ir] / tc[ic]:6.2f}", flush=True)
    print("SR-PR: R-MAT (a,b,c)=(0.45,0.22,0.22), 16 entries per row, N = 32")
    for i, scale in enumerate((10, 12, 14, 17, 20)):
        m = gen.rmat_csr(scale, 16.0, 0.45, 0.22, 0.22, seed=8220 + i)
        line(f"  scale {scale}: {m.m} rows, {m.nnz} entries", time_all(m, 32), SR, PR, "SR", "PR")


if __name__ == "__main__":
    sys.exit(main())
