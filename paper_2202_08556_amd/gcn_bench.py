"""GCN aggregation as a second workload (the application of the paper's Sec. 6): forward A.X and
backward A^T.dY on the power-law graph of the headline benchmark, feature lengths 16 ... 256.

    python -m paper_2202_08556_amd.gcn_bench [--m 262144] [--out results/gcn_bench.txt]

For every feature length: time of each of the 8 algorithm ids and of the selector's choice, for
A (forward) and for A^T (backward); the one-off cost of da_csr_transpose; and one two-layer GCN
inference pass (relu(A.(X.W1)) -> A.(H.W2)) with the dense products in the GEMM library.
Times are HIP-event times over back-to-back calls that rotate over 3 copies of the dense operands.
"""
from __future__ import annotations

import argparse
import sys

import numpy as np
import torch

from . import binding as da
from . import gcn
from . import generators as gen
from .sweep import time_algo

NS = (16, 32, 64, 128, 256)
COPIES = 3


def time_all(graph: gcn.SparseGraph, N: int, seed: int):
    dev = graph.rowptr.device
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    Bs = [torch.empty((graph.k, N), device=dev).normal_(generator=g) for _ in range(COPIES)]
    Cs = [torch.empty((graph.m, N), device=dev) for _ in range(COPIES)]
    graph.spmm(Bs[0])                               # makes sure the matrix is prepared
    runs = [da.PreparedSpmm(graph.m, graph.k, N, graph.rowptr, graph.colind, graph.vals, Bs[i], Cs[i])
            for i in range(COPIES)]
    times = []
    for algo in range(da.DA_NUM_ALGOS):
        t, _ = time_algo(lambda i, algo=algo: runs[i % COPIES](algo))
        times.append(t)
    return times


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--m", type=int, default=262144)
    ap.add_argument("--seed", type=int, default=gen.config_seed(2))
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
    a = gen.powerlaw_csr(m=args.m, seed=args.seed)
    from .profile_summary import source_hash
    lines = ["GCN aggregation on the power-law graph: forward A.X, backward A^T.dY, all 8 ids vs the selector's choice,",
             "one-off da_csr_transpose, two-layer GCN inference.  MI355X, HIP-event times (us); both matrices prepared",
             "with da_spmm_prepare (EB chunk schedule).",
             "command (repository root, after __graft_entry__.build()): python -m paper_2202_08556_amd.gcn_bench --out FILE",
             f"SOURCE_SHA256 = {source_hash()}",
             "ids in the last column, in order: " + " ".join(da.ALGO_NAMES),
             f"power-law graph m=k={a.m} nnz={a.nnz} seed={args.seed} (values 1/row length: row-normalised adjacency)"]
    graph = gcn.SparseGraph.from_numpy(a)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    tt = []
    for rep in range(4):
        graph._t = None
        e0.record()
        graph.transposed()
        e1.record()
        torch.cuda.synchronize()
        tt.append(e0.elapsed_time(e1) * 1e3)
    lines.append(f"da_csr_transpose (incl. workspace allocation): first {tt[0]:.0f} us, then {min(tt[1:]):.0f} us")
    gt = graph.transposed()
    for label, gr in (("forward  A.X   ", graph), ("backward A^T.dY", gt)):
        f = gr.features(1)
        lines.append(f"{label}: rows {f['rows']} mean row {f['row_nnz_mean']:.1f} std {f['row_nnz_std']:.1f} "
                     f"max {f['row_nnz_max']:.0f}")
    lines.append("N    direction  chosen      t_chosen_us  best        t_best_us  chosen/best  GFLOP/s(chosen)   all 8 ids (us)")
    ratios = []
    for N in NS:
        for label, gr in (("fwd", graph), ("bwd", gt)):
            times = time_all(gr, N, args.seed + N)
            ch = gr.algo_for(N)
            best = int(np.argmin(times))
            ratios.append(times[best] / times[ch])
            lines.append(f"{N:<4d} {label}        {da.ALGO_NAMES[ch]:<10s}  {times[ch]:11.1f}  {da.ALGO_NAMES[best]:<10s}  "
                         f"{times[best]:9.1f}  {times[ch] / times[best]:11.3f}  {2.0 * a.nnz * N / times[ch] / 1e3:15.1f}   "
                         + " ".join(f"{t:.0f}" for t in times))
            print(lines[-1], flush=True)
    lines.append(f"selector normalised performance over these {len(ratios)} points (geometric mean of best/chosen): "
                 f"{float(np.exp(np.mean(np.log(ratios)))):.4f}")
    # two-layer GCN inference, hidden width 128, 602 input features and 41 classes as in the
    # citation-style node classification setting the paper's experiment uses
    fin, hid, ncls = 602, 128, 41
    dev = graph.rowptr.device
    torch.manual_seed(0)
    X = torch.randn((a.m, fin), device=dev)
    l1, l2 = gcn.GraphConv(fin, hid).to(dev), gcn.GraphConv(hid, ncls, relu=False).to(dev)
    with torch.no_grad():
        def infer(_i):
            return l2(graph, l1(graph, X))
        t, reps = time_algo(infer, budget_ms=50.0)
        e0.record()
        for _ in range(5):
            H = X @ l1.weight
            H2 = torch.relu(H) @ l2.weight
        e1.record()
        torch.cuda.synchronize()
        dense_us = e0.elapsed_time(e1) / 5 * 1e3
    lines.append(f"two-layer GCN inference ({fin}->{hid}->{ncls}): {t:.0f} us per pass, of which about {dense_us:.0f} us "
                 f"are the two dense products; aggregation ids: N={hid} {da.ALGO_NAMES[graph.algo_for(hid)]}, "
                 f"N={ncls} {da.ALGO_NAMES[graph.algo_for(ncls)]}")
    text = "\n".join(lines)
    print(text)
    if args.out:
        open(args.out, "w").write(text + "\n")


if __name__ == "__main__":
    sys.exit(main())
