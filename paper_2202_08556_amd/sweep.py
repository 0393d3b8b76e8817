"""Time all 8 algorithm ids on families of seeded matrices: the data the selector is trained and
scored on (paper Sec. 5: every design is run on every matrix, the model learns which one wins).

    python -m paper_2202_08556_amd.sweep --set eval  --members 0-63  --out results/sweep_eval.jsonl
    python -m paper_2202_08556_amd.sweep --set train --members 0-255 --out results/sweep_train.jsonl
    python -m paper_2202_08556_amd.sweep --set families --out results/sweep_families.jsonl
    python -m paper_2202_08556_amd.sweep --set odd --out results/sweep_odd.jsonl

Sets
  eval      the 64-member selector sweep (seed base 5000), never trained on
  train     members of the same lognormal family with a disjoint seed base (100000) and a lower
            size cap (2^24 entries), used for training only
  families  scaled versions of the uniform / power-law / stencil / skewed workloads with seeds
            disjoint from the benchmark configurations, plus odd shapes (see odd_members), used
            for training only
  odd       other members of those odd shapes (different sizes and seeds), never trained on

--ns 2,4 runs the same matrices at other dense widths (the paper also reports N = 2).

One JSON line per (matrix, N): features as returned by da_spmm_features, and the time of each id
in microseconds (HIP events around a batch of back-to-back calls that rotate over 3 copies of B
and C).  Points already present in the output file are skipped, so a run can be resumed.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

from . import binding as da
from . import generators as gen

NS = (8, 16, 32, 64, 128, 256)
COPIES = 3


def parse_members(spec: str):
    out = []
    for part in spec.split(","):
        if "-" in part:
            a, b = part.split("-")
            out.extend(range(int(a), int(b) + 1))
        else:
            out.append(int(part))
    return out


def family_members():
    """(name, constructor) pairs; seeds 7000+ are used nowhere else."""
    fam = []
    for i, m in enumerate((4096, 16384, 65536, 262144)):
        fam.append((f"uniform_m{m}", lambda m=m, i=i: gen.uniform_csr(m=m, k=m, mean_len=8.0, seed=7000 + i)))
        fam.append((f"uniform32_m{m}", lambda m=m, i=i: gen.uniform_csr(m=m, k=m, mean_len=32.0, seed=7010 + i)))
    for i, m in enumerate((8192, 32768, 131072, 262144)):
        fam.append((f"powerlaw_m{m}", lambda m=m, i=i: gen.powerlaw_csr(m=m, seed=7100 + i)))
        fam.append((f"powerlaw_s2_m{m}", lambda m=m, i=i: gen.powerlaw_csr(m=m, scale=2.0, max_len=1024, seed=7110 + i)))
    for i, g in enumerate(((16, 16, 16), (32, 32, 32), (64, 64, 64), (48, 96, 128), (64, 128, 96))):
        fam.append((f"stencil_{g[0]}x{g[1]}x{g[2]}", lambda g=g, i=i: gen.stencil27_csr(*g, seed=7200 + i)))
    for i, (m, lo, hi) in enumerate(((16384, 2000, 8000), (65536, 5000, 30000), (262144, 20000, 100000),
                                     (524288, 10000, 50000))):
        fam.append((f"skewed_m{m}", lambda m=m, lo=lo, hi=hi, i=i: gen.skewed_csr(m=m, heavy_lo=lo, heavy_hi=hi,
                                                                               seed=7300 + i)))
    # in-link matrices of power-law graphs (a GNN's backward pass) and R-MAT graphs
    for i, m in enumerate((16384, 65536, 262144)):
        fam.append((f"powerlaw_rev_m{m}", lambda m=m, i=i: gen.reversed_edges(gen.powerlaw_csr(m=m, seed=7400 + i))))
    for i, (scale, ef, a, b) in enumerate(((14, 16.0, 0.57, 0.19), (16, 16.0, 0.57, 0.19), (18, 16.0, 0.57, 0.19),
                                           (16, 32.0, 0.45, 0.15), (17, 8.0, 0.65, 0.15))):
        fam.append((f"rmat_s{scale}_e{int(ef)}_a{int(a * 100)}",
                    lambda scale=scale, ef=ef, a=a, b=b, i=i: gen.rmat_csr(scale, ef, a, b, b, seed=7500 + i)))
    fam.extend(odd_members(7600, train=True))
    return fam


def odd_members(seed0: int, train: bool):
    """Shapes far from the lognormal family: nearly all rows empty, about one entry per row, a few
    very long rows in a wide matrix, millions of short rows over few columns, single dense rows.
    The training members (train=True) and the evaluation members differ in sizes and seeds."""
    if train:
        hyper = ((1 << 20, 0.01, 100.0), (1 << 22, 0.001, 500.0), (1 << 21, 0.1, 8.0), (1 << 23, 0.0002, 4.0))
        short = ((1 << 21, 1 << 21, 1.0), (1 << 22, 1 << 19, 0.5))
        wide = ((2000, 1 << 22, 5000.0), (500, 1 << 20, 20000.0))
        tall = ((6_000_000, 2000, 3.0), (2_000_000, 500, 6.0))
        dense_rows = ((300_000, 1, 250_000, 8.0), (100_000, 5, 80_000, 2.0))
    else:
        hyper = ((3_000_000, 0.005, 60.0), (6_000_000, 0.0005, 300.0))
        short = ((3_000_000, 3_000_000, 1.5),)
        wide = ((1000, 2_000_000, 8000.0),)
        tall = ((4_000_000, 1000, 4.0),)
        dense_rows = ((200_000, 2, 150_000, 6.0),)
    fam = []
    for i, (m, frac, mean) in enumerate(hyper):
        fam.append((f"hypersparse_m{m}_f{frac}", lambda m=m, frac=frac, mean=mean, i=i:
                    gen.hypersparse_csr(m, m // 8, frac, mean, seed=seed0 + i)))
    for i, (m, k, mean) in enumerate(short):
        fam.append((f"short_m{m}_k{k}", lambda m=m, k=k, mean=mean, i=i: gen.uniform_csr(m, k, mean, seed=seed0 + 10 + i)))
    for i, (m, k, mean) in enumerate(wide):
        fam.append((f"wide_m{m}_k{k}", lambda m=m, k=k, mean=mean, i=i: gen.uniform_csr(m, k, mean, seed=seed0 + 20 + i)))
    for i, (m, k, mean) in enumerate(tall):
        fam.append((f"tall_m{m}_k{k}", lambda m=m, k=k, mean=mean, i=i: gen.uniform_csr(m, k, mean, seed=seed0 + 30 + i)))
    for i, (m, rows, length, light) in enumerate(dense_rows):
        fam.append((f"denserows_m{m}_r{rows}", lambda m=m, rows=rows, length=length, light=light, i=i:
                    gen.skewed_csr(m=m, heavy_frac=rows / m, heavy_lo=length, heavy_hi=length, light_mean=light,
                                   seed=seed0 + 40 + i)))
    return fam


def time_algo(call, first_only_above_ms=40.0, budget_ms=8.0, max_reps=30):
    """Median-free simple protocol: one warm-up, then a batch sized to ~budget_ms, events around it."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    call(0)
    torch.cuda.synchronize()
    e0.record()
    call(1)
    e1.record()
    torch.cuda.synchronize()
    t1 = e0.elapsed_time(e1)
    if t1 > first_only_above_ms:
        return t1 * 1e3, 1
    reps = int(max(3, min(max_reps, budget_ms / max(t1, 1e-3))))
    e0.record()
    for i in range(reps):
        call(2 + i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps * 1e3, reps


def run_matrix(a, tag, member, setname, out, done, ns=NS):
    dev = torch.device("cuda:0")
    rp = torch.from_numpy(a.rowptr).to(dev)
    ci = torch.from_numpy(a.colind).to(dev)
    va = torch.from_numpy(a.vals).to(dev)
    # the per-matrix preparation a user of the EB ids would do once (chunk order); the timings below
    # are those of a prepared matrix
    da.da_spmm_prepare(a.m, a.k, a.nnz, rp, ci)
    for N in ns:
        key = (setname, tag, N)
        if key in done:
            continue
        feats = da.da_spmm_features(a.m, N, rp)
        g = torch.Generator(device=dev)
        g.manual_seed(a.seed * 1000 + N)
        Bs = [torch.empty((a.k, N), device=dev).uniform_(-1.0, 1.0, generator=g) for _ in range(COPIES)]
        Cs = [torch.empty((a.m, N), device=dev) for _ in range(COPIES)]
        times, reps = [], []
        runs = [da.PreparedSpmm(a.m, a.k, N, rp, ci, va, Bs[i], Cs[i]) for i in range(COPIES)]
        for algo in range(da.DA_NUM_ALGOS):
            def call(i, algo=algo):
                runs[i % COPIES](algo)
            t, r = time_algo(call)
            times.append(round(t, 2))
            reps.append(r)
        rec = dict(set=setname, name=tag, member=member, seed=a.seed, m=a.m, k=a.k, nnz=a.nnz, N=N,
                   features=feats, times_us=times, reps=reps)
        out.write(json.dumps(rec) + "\n")
        out.flush()
        best = int(np.argmin(times))
        print(f"{setname} {tag} N={N}: best {da.ALGO_NAMES[best]} {times[best]:.1f} us  " +
              " ".join(f"{t:.0f}" for t in times), flush=True)
        del runs, Bs, Cs
    da.da_spmm_release(rp)
    del rp, ci, va


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--set", default="eval", choices=["eval", "train", "families", "odd"])
    ap.add_argument("--members", default=None)
    ap.add_argument("--out", required=True)
    ap.add_argument("--max-seconds", type=float, default=1e9, help="stop starting new matrices after this")
    ap.add_argument("--ns", default=None, help="comma-separated dense widths instead of 8,16,32,64,128,256")
    args = ap.parse_args()
    ns = tuple(int(x) for x in args.ns.split(",")) if args.ns else NS
    done = set()
    if os.path.exists(args.out):
        for line in open(args.out):
            try:
                r = json.loads(line)
                done.add((r["set"], r["name"], r["N"]))
            except ValueError:
                pass
    t0 = time.time()
    with open(args.out, "a") as out:
        if args.set in ("families", "odd"):
            members = family_members() if args.set == "families" else odd_members(7800, train=False)
            for idx, (name, make) in enumerate(members):
                if all((args.set, name, N) in done for N in ns):
                    continue
                if time.time() - t0 > args.max_seconds:
                    break
                run_matrix(make(), name, idx, args.set, out, done, ns)
        else:
            base, cap = (5000, 2 ** 26) if args.set == "eval" else (100000, 2 ** 24)
            members = parse_members(args.members or ("0-63" if args.set == "eval" else "0-255"))
            for j in members:
                tag = f"sweep{j}"
                if all((args.set, tag, N) in done for N in ns):
                    continue
                if time.time() - t0 > args.max_seconds:
                    break
                m, mean_len, cv, seed = gen.sweep_params(j, base, cap)
                a = gen.lognormal_csr(m, mean_len, cv, seed, name=tag)
                run_matrix(a, tag, j, args.set, out, done, ns)
    print("sweep finished", flush=True)


if __name__ == "__main__":
    sys.exit(main())
