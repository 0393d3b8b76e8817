"""rocprofv3 harness: runs the profiler over bench.py and reduces its output to the short text
summaries kept under profiles/ (achieved HBM traffic against the MI355X peak, Sec. 6 style
measurement of the kernels).

    python -m paper_2202_08556_amd.profile_summary run --workload powerlaw --N 128 [--out-dir gpurun_out/profiles]
        six rocprofv3 passes, each a run of its own (counters are never combined with traces):
          1. --kernel-trace --stats  over `python3 bench.py --workload W --N n`      -> per-kernel durations
          2. --pmc FETCH_SIZE        over a short bench run                           -> KiB fetched per dispatch
          3. --pmc WRITE_SIZE        over a short bench run                           -> KiB written per dispatch
          4. --pmc TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum                               -> L2 hit rate
          5./6. FETCH_SIZE / WRITE_SIZE over the plain copy kernel `calib_copy 1024`  -> counter scale factors
        and then the two reductions below.
    python -m paper_2202_08556_amd.profile_summary kernel-trace DIR --bench-json FILE --out FILE --command TEXT
    python -m paper_2202_08556_amd.profile_summary hbm-traffic --fetch DIR --write DIR --tcc DIR
                          --calib-fetch DIR --calib-write DIR --bench-json FILE --out FILE --command TEXT
    python -m paper_2202_08556_amd.profile_summary bench-configs [--out FILE]
        bench.py once per named configuration; one JSON line each.

The parent process never touches the GPU: the profiler and bench.py run as child processes, each
under a time limit, and a failing pass ends the run.

Every summary carries SOURCE_SHA256, the hash of the kernel sources it was measured on
(source_hash()), and the machine-readable lines bench.py reads back; bench.py reports a summary's
traffic only when that hash equals the hash of the sources it runs on.
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import sqlite3
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CALIB_MIB = 1024


def source_hash() -> str:
    """sha256 over the HIP / C++ sources of libdaspmm.so and the header (names and contents)."""
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(PKG, "csrc", "*.hip")) + glob.glob(os.path.join(PKG, "csrc", "*.cpp")) +
                   glob.glob(os.path.join(PKG, "csrc", "*.inc")) + glob.glob(os.path.join(ROOT, "include", "*.h")))
    for f in files:
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def git_head() -> str:
    try:
        return subprocess.check_output(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], text=True,
                                       stderr=subprocess.DEVNULL).strip()
    except Exception:
        return "unknown (no git metadata where the run took place)"


def find_db(directory: str) -> str:
    hits = sorted(glob.glob(os.path.join(directory, "**", "*_results.db"), recursive=True))
    if not hits:
        raise SystemExit(f"no rocprofv3 result database under {directory}")
    return hits[-1]


def short_name(kernel: str) -> str:
    """`void daspmm::eb_sr_kernel<4, 32, 1, false>(int, ...)` -> `daspmm::eb_sr_kernel<4, 32, 1, false>`."""
    name = kernel.split("(")[0].strip()
    return name[5:] if name.startswith("void ") else name


def kernel_rows(db_path: str):
    """[(name, calls, avg_us, min_us, max_us, total_us)] by total time, from the kernel trace."""
    db = sqlite3.connect(db_path)
    rows = db.execute("select name, count(*), avg(end-start), min(end-start), max(end-start), sum(end-start) "
                      "from kernels group by name order by sum(end-start) desc").fetchall()
    return [(short_name(r[0]), int(r[1]), r[2] / 1e3, r[3] / 1e3, r[4] / 1e3, r[5] / 1e3) for r in rows]


def counter_rows(db_path: str):
    """[(kernel, counter, dispatches, average value per dispatch)] from a --pmc run."""
    db = sqlite3.connect(db_path)
    rows = db.execute("select kernel_name, counter_name, count(*), avg(value) from counters_collection "
                      "group by kernel_name, counter_name").fetchall()
    return [(short_name(r[0]), r[1], int(r[2]), float(r[3])) for r in rows]


def bench_line(path: str) -> dict:
    with open(path) as fh:
        lines = [l for l in fh.read().strip().splitlines() if l.startswith("{")]
    return json.loads(lines[-1])


def product_kernels(names, algo: str):
    """The kernels one da_spmm call of the algorithm family launches: the main kernel that ran most
    often in the timed region, plus the EB zero pre-pass."""
    fam = {"RB": "rb", "EB": "eb"}[algo[:2]] + "_" + {"SR": "sr", "PR": "pr"}[algo[-2:]] + "_kernel"
    return [n for n in names if fam in n or (algo.startswith("EB") and "eb_zero_kernel" in n)]


def write_kernel_trace(trace_dir: str, bench_json: str, out: str, command: str) -> dict:
    bench = bench_line(bench_json)
    rows = kernel_rows(find_db(trace_dir))
    total = sum(r[5] for r in rows) or 1.0
    algo = bench["config"]["algo"]
    mains = [r for r in rows if r[0] in product_kernels([r[0] for r in rows], algo)]
    # the timed region dominates the call counts: the instantiation of the chosen family with the most calls
    main = max((r for r in mains if "eb_zero" not in r[0]), key=lambda r: r[1])
    zero = max((r for r in mains if "eb_zero" in r[0]), key=lambda r: r[1], default=None)
    per_call = main[2] + (zero[2] if zero else 0.0)
    lines = [f"rocprofv3 kernel-trace summary: {bench['config']['workload']}",
             "command (from the repository root, after __graft_entry__.build()):", f"  {command}",
             f"GIT_HEAD = {git_head()}", f"SOURCE_SHA256 = {source_hash()}",
             "per-kernel aggregate of the `kernels` view of the result database (durations end-start, microseconds)", "",
             f"{'kernel':74s} {'calls':>6s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'pct':>6s}"]
    for r in rows[:16]:
        lines.append(f"{r[0][:74]:74s} {r[1]:6d} {r[2]:10.2f} {r[3]:10.2f} {r[4]:10.2f} {100 * r[5] / total:6.2f}")
    lines += ["", f"ALGO = {algo}", f"MAIN_KERNEL = {main[0]}", f"MAIN_KERNEL_AVG_US = {main[2]:.2f}",
              f"ZERO_KERNEL_AVG_US = {zero[2]:.2f}" if zero else "ZERO_KERNEL_AVG_US = 0",
              f"KERNEL_US_PER_CALL = {per_call:.2f}",
              f"BENCH_US_PER_STEP = {bench['ms_per_step'] * 1e3:.2f}   (HIP events inside bench.py, same run)",
              "The radix_* / scan_* / schedule_* kernels belong to da_spmm_prepare (once per matrix copy, outside the",
              "timed region); other product kernels are the per-algorithm timing passes bench.py makes before it.",
              "bench.py line of the same run:", json.dumps(bench), ""]
    os.makedirs(os.path.dirname(os.path.abspath(out)), exist_ok=True)
    with open(out, "w") as fh:
        fh.write("\n".join(lines))
    return {"kernel_us_per_call": per_call, "main": main[0]}


def write_hbm_traffic(fetch: str, write: str, tcc: str | None, calib_fetch: str, calib_write: str, bench_json: str,
                      out: str, command: str, us_per_call: float | None = None) -> dict:
    bench = bench_line(bench_json)
    algo = bench["config"]["algo"]
    cfg = bench["config"]
    calib_kib = CALIB_MIB * 1024.0

    def calib_scale(directory, counter):
        vals = [v for (k, c, n, v) in counter_rows(find_db(directory)) if c == counter and "calib_copy_kernel" in k]
        if not vals:
            raise SystemExit(f"no {counter} reading of calib_copy_kernel under {directory}")
        return calib_kib / vals[0], vals[0]

    sf, rf = calib_scale(calib_fetch, "FETCH_SIZE")
    sw, rw = calib_scale(calib_write, "WRITE_SIZE")

    def per_call(directory, counter):
        rows = [r for r in counter_rows(find_db(directory)) if r[1] == counter]
        names = product_kernels([r[0] for r in rows], algo)
        mains = [r for r in rows if r[0] in names and "eb_zero" not in r[0]]
        zeros = [r for r in rows if r[0] in names and "eb_zero" in r[0]]
        main = max(mains, key=lambda r: r[2])
        zero = max(zeros, key=lambda r: r[2], default=None)
        return main, zero, rows

    fmain, fzero, frows = per_call(fetch, "FETCH_SIZE")
    wmain, wzero, wrows = per_call(write, "WRITE_SIZE")
    F = sf * (fmain[3] + (fzero[3] if fzero else 0.0))
    W = sw * (wmain[3] + (wzero[3] if wzero else 0.0))
    m, k, nnz, N = cfg["m"], cfg["k"], cfg["nnz"], cfg["N"]
    read_comp = 4 * (m + 1) + 8 * nnz + 4 * k * N
    write_comp = 4 * m * N
    # time of an un-instrumented call: the kernel-trace figure when given (counter collection slows
    # the kernels down), else this run's own step time
    us = us_per_call if us_per_call else bench["ms_per_step"] * 1e3
    us_src = "kernel-trace run of the same command" if us_per_call else "bench.py step time of the counter run itself, inflated by the counters"
    lines = [f"rocprofv3 HBM traffic counters: {cfg['workload']} ({algo})",
             "commands (one counter set per run; from the repository root, after __graft_entry__.build()):"]
    lines += [f"  {c}" for c in command.split("\n")]
    lines += [f"GIT_HEAD = {git_head()}", f"SOURCE_SHA256 = {source_hash()}",
              "values = average per dispatch of the `counters_collection` view (FETCH_SIZE / WRITE_SIZE in KiB)", ""]
    shown = {fmain[0], fzero[0] if fzero else ""}
    for (kname, c, n, v) in frows + wrows:
        if kname in shown:
            lines.append(f"{kname[:70]:70s} {c:12s} dispatches={n:4d} avg_per_dispatch={v:.6g}")
    hit = None
    if tcc:
        trows = counter_rows(find_db(tcc))
        t = {c: v for (kname, c, n, v) in trows if kname == fmain[0]}
        for (kname, c, n, v) in trows:
            if kname in shown:
                lines.append(f"{kname[:70]:70s} {c:12s} dispatches={n:4d} avg_per_dispatch={v:.6g}")
        if t.get("TCC_REQ_sum"):
            hit = t["TCC_HIT_sum"] / t["TCC_REQ_sum"]
    lines += ["", f"calibration: plain copy kernel, {CALIB_MIB} MiB read + {CALIB_MIB} MiB written per dispatch ({calib_kib:.0f} KiB each)",
              f"  FETCH_SIZE reads {rf:.6g} -> scale {sf:.3f}; WRITE_SIZE reads {rw:.6g} -> scale {sw:.3f}", "",
              "per da_spmm call (main kernel + EB zero pre-pass), scaled:",
              f"ALGO = {algo}", f"MAIN_KERNEL = {fmain[0]}",
              f"FETCH_KIB_PER_CALL_SCALED = {F:.0f}", f"WRITE_KIB_PER_CALL_SCALED = {W:.0f}",
              f"TCC_HIT_RATE = {hit:.4f}" if hit is not None else "TCC_HIT_RATE = n/a",
              f"  read  {F * 1024 / 1e9:.3f} GB = {F * 1024 / read_comp:.2f} x the compulsory read bytes (CSR + B once = {read_comp / 1e6:.1f} MB)",
              f"  write {W * 1024 / 1e9:.3f} GB = {W * 1024 / write_comp:.2f} x the compulsory written bytes (C once = {write_comp / 1e6:.1f} MB)",
              f"  ({F * 1024 / 1e9:.3f} + {W * 1024 / 1e9:.3f}) GB / {us:.1f} us ({us_src}) = "
              f"{(F + W) * 1024 / 1e9 / (us * 1e-6) / 1e3:.2f} TB/s through the L2-to-fabric interface",
              "bench.py line of the FETCH_SIZE run:", json.dumps(bench), ""]
    os.makedirs(os.path.dirname(os.path.abspath(out)), exist_ok=True)
    with open(out, "w") as fh:
        fh.write("\n".join(lines))
    return {"fetch_bytes": F * 1024, "write_bytes": W * 1024, "hit": hit}


def read_summary(path: str) -> dict:
    """KEY = value lines of a summary written by this module."""
    vals = {}
    try:
        with open(path) as fh:
            for line in fh:
                if " = " in line and line.split(" = ")[0].strip().replace("_", "").isalnum() and line[0].isupper():
                    key, v = line.split(" = ", 1)
                    vals[key.strip()] = v.strip()
    except OSError:
        pass
    return vals


def _run(cmd, log, limit):
    print("+", " ".join(cmd), flush=True)
    env = dict(os.environ, TMPDIR="/tmp")
    with open(log, "w") as fh:
        try:
            rc = subprocess.run(cmd, stdout=fh, stderr=subprocess.STDOUT, cwd=ROOT, env=env, timeout=limit).returncode
        except subprocess.TimeoutExpired:
            raise SystemExit(f"time limit of {limit} s exceeded: {' '.join(cmd)} (see {log})")
    if rc != 0:
        raise SystemExit(f"exit status {rc}: {' '.join(cmd)} (see {log})")


def run_all(workload: str, N: int, out_dir: str, raw_dir: str, extra):
    """The six profiler passes and both reductions for one workload."""
    tag = f"{workload}_N{N}"
    os.makedirs(raw_dir, exist_ok=True)
    # without the extra pass over unprepared matrices: every call of the chosen kernel is then one of
    # the calls the benchmark times, and the trace's average can be compared with the benchmark's
    bench = ["python3", "bench.py", "--workload", workload, "--N", str(N), "--no-unprepared", *extra]
    short = [*bench, "--no-variants", "--no-cpu-baseline", "--steps", "10", "--warmup", "2"]
    calib = [os.path.join(PKG, "calib_copy"), str(CALIB_MIB)]

    def prof(kind, args, target, limit, json_out=None):
        d = os.path.join(raw_dir, f"{kind}_{tag}")
        subprocess.run(["rm", "-rf", d])
        cmd = ["rocprofv3", *args, "-d", d, "-o", "run", "--", *target]
        log = d + ".log"
        _run(cmd, log, limit)
        if json_out:
            with open(log) as fh, open(json_out, "w") as jo:
                jo.write("\n".join(l for l in fh.read().splitlines() if l.startswith("{")) + "\n")
        return d, " ".join(cmd).replace(ROOT + "/", "")

    cmds = []
    tj = os.path.join(raw_dir, f"trace_{tag}.json")
    td, c = prof("trace", ["--kernel-trace", "--stats"], bench, 600, tj)
    kt = write_kernel_trace(td, tj, os.path.join(out_dir, f"da_spmm_{tag}_kernel_trace.txt"), c)
    fj = os.path.join(raw_dir, f"fetch_{tag}.json")
    fd, c = prof("fetch", ["--pmc", "FETCH_SIZE"], short, 300, fj); cmds.append(c)
    wd, c = prof("write", ["--pmc", "WRITE_SIZE"], short, 300); cmds.append(c)
    cd, c = prof("tcc", ["--pmc", "TCC_HIT_sum", "TCC_MISS_sum", "TCC_REQ_sum"], short, 300); cmds.append(c)
    cfd, c = prof("calibfetch", ["--pmc", "FETCH_SIZE"], calib, 120); cmds.append(c)
    cwd, c = prof("calibwrite", ["--pmc", "WRITE_SIZE"], calib, 120); cmds.append(c)
    res = write_hbm_traffic(fd, wd, cd, cfd, cwd, fj, os.path.join(out_dir, f"da_spmm_{tag}_hbm_traffic.txt"), "\n".join(cmds),
                            kt["kernel_us_per_call"])
    print(json.dumps({"workload": tag, **res}), flush=True)


NAMED_CONFIGS = [("uniform", 8), ("powerlaw", 32), ("powerlaw", 128), ("stencil", 32), ("skewed", 8), ("skewed", 64)]


def bench_configs(out: str):
    lines = [f"bench.py on every named configuration (one JSON line each); GIT_HEAD = {git_head()}",
             f"SOURCE_SHA256 = {source_hash()}",
             "command per line: python3 bench.py --workload W --N n --steps 100 --warmup 10"]
    for (w, n) in NAMED_CONFIGS:
        cmd = ["python3", "bench.py", "--workload", w, "--N", str(n), "--steps", "100", "--warmup", "10"]
        print("+", " ".join(cmd), flush=True)
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True, cwd=ROOT, timeout=600)
        if res.returncode != 0:
            raise SystemExit(f"exit status {res.returncode}: {' '.join(cmd)}")
        lines.append([l for l in res.stdout.splitlines() if l.startswith("{")][-1])
    os.makedirs(os.path.dirname(os.path.abspath(out)), exist_ok=True)
    with open(out, "w") as fh:
        fh.write("\n".join(lines) + "\n")


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    r = sub.add_parser("run")
    r.add_argument("--workload", default="powerlaw")
    r.add_argument("--N", type=int, default=128)
    r.add_argument("--out-dir", default=os.path.join(ROOT, "gpurun_out", "profiles"))
    r.add_argument("--raw-dir", default=os.path.join(ROOT, "gpurun_out", "rocprof"))
    r.add_argument("bench_args", nargs="*", help="further arguments for bench.py (after --)")
    k = sub.add_parser("kernel-trace")
    k.add_argument("dir")
    k.add_argument("--bench-json", required=True)
    k.add_argument("--out", required=True)
    k.add_argument("--command", default="rocprofv3 --kernel-trace --stats -d DIR -o run -- python3 bench.py")
    h = sub.add_parser("hbm-traffic")
    for name in ("fetch", "write", "calib-fetch", "calib-write"):
        h.add_argument("--" + name, required=True)
    h.add_argument("--tcc")
    h.add_argument("--bench-json", required=True)
    h.add_argument("--out", required=True)
    h.add_argument("--us-per-call", type=float, default=None)
    h.add_argument("--command", default="rocprofv3 --pmc COUNTER -d DIR -o run -- python3 bench.py --no-variants --no-cpu-baseline --steps 10 --warmup 2")
    b = sub.add_parser("bench-configs")
    b.add_argument("--out", default=os.path.join(ROOT, "gpurun_out", "profiles", "bench_named_configs.txt"))
    sub.add_parser("source-hash")
    a = ap.parse_args(argv)
    if a.cmd == "run":
        run_all(a.workload, a.N, a.out_dir, a.raw_dir, a.bench_args)
    elif a.cmd == "kernel-trace":
        write_kernel_trace(a.dir, a.bench_json, a.out, a.command)
    elif a.cmd == "hbm-traffic":
        write_hbm_traffic(a.fetch, a.write, a.tcc, a.calib_fetch, a.calib_write, a.bench_json, a.out, a.command,
                          a.us_per_call)
    elif a.cmd == "bench-configs":
        bench_configs(a.out)
    else:
        print(source_hash())


if __name__ == "__main__":
    main()
