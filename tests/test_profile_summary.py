"""Host logic of the rocprofv3 harness (paper_2202_08556_amd.profile_summary): the reduction of a
profiler result database to the summaries under profiles/, checked on small databases built here
with the two views the harness reads, and the rule bench.py uses to accept a summary."""
import json
import os
import sqlite3

import pytest

from paper_2202_08556_amd import profile_summary as ps

EB = "void daspmm::eb_sr_kernel<4, 32, 1, false>(int, int, daspmm::Strides, int const*)"
ZERO = "void daspmm::eb_zero_kernel<4>(int, int, daspmm::Strides, int const*, float*, int, int)"
OTHER = "void daspmm::rb_sr_kernel<4, 32, 1, false>(int, int)"
COPY = "calib_copy_kernel(float4 const*, float4*, unsigned long)"


def make_db(directory, kernels=(), counters=()):
    os.makedirs(directory, exist_ok=True)
    db = sqlite3.connect(os.path.join(directory, "run_results.db"))
    db.execute("create table kernels (name text, start integer, end integer)")
    db.execute("create table counters_collection (kernel_name text, counter_name text, value real, duration integer)")
    db.executemany("insert into kernels values (?, ?, ?)", kernels)
    db.executemany("insert into counters_collection values (?, ?, ?, 0)", counters)
    db.commit()
    db.close()


def bench_json(path, algo="EB+RM+SR", ms=0.5):
    line = {"ms_per_step": ms, "config": {"workload": "test workload", "algo": algo, "m": 1000, "k": 1000, "nnz": 50000, "N": 128}}
    with open(path, "w") as fh:
        fh.write("some log line\n" + json.dumps(line) + "\n")
    return line


def test_short_name_and_product_kernels():
    assert ps.short_name(EB) == "daspmm::eb_sr_kernel<4, 32, 1, false>"
    names = [ps.short_name(x) for x in (EB, ZERO, OTHER)]
    assert ps.product_kernels(names, "EB+RM+SR") == names[:2]
    assert ps.product_kernels(names, "RB+RM+SR") == names[2:]


def test_kernel_trace_summary(tmp_path):
    d = str(tmp_path / "trace")
    rows = [(EB, 0, 400_000)] * 3 + [(EB, 0, 500_000)] + [(ZERO, 0, 6_000)] * 4 + [(OTHER, 0, 900_000)]
    make_db(d, kernels=rows)
    bj = str(tmp_path / "b.json")
    bench_json(bj)
    out = str(tmp_path / "kt.txt")
    res = ps.write_kernel_trace(d, bj, out, "rocprofv3 --kernel-trace --stats -- python3 bench.py")
    assert res["kernel_us_per_call"] == pytest.approx(425.0 + 6.0)
    vals = ps.read_summary(out)
    assert vals["ALGO"] == "EB+RM+SR"
    assert float(vals["MAIN_KERNEL_AVG_US"]) == pytest.approx(425.0)
    assert float(vals["ZERO_KERNEL_AVG_US"]) == pytest.approx(6.0)
    assert vals["SOURCE_SHA256"] == ps.source_hash()


def test_hbm_traffic_summary_scales_by_the_copy_kernel(tmp_path):
    mib = ps.CALIB_MIB * 1024.0
    # the fetch counter reads half of the copied KiB (scale 2), the write counter all of it (scale 1)
    make_db(str(tmp_path / "cf"), counters=[(COPY, "FETCH_SIZE", mib / 2)])
    make_db(str(tmp_path / "cw"), counters=[(COPY, "WRITE_SIZE", mib)])
    make_db(str(tmp_path / "f"), counters=[(EB, "FETCH_SIZE", 1000.0), (EB, "FETCH_SIZE", 3000.0), (ZERO, "FETCH_SIZE", 10.0),
                                            (OTHER, "FETCH_SIZE", 7.0)])
    make_db(str(tmp_path / "w"), counters=[(EB, "WRITE_SIZE", 500.0), (ZERO, "WRITE_SIZE", 20.0)])
    make_db(str(tmp_path / "t"), counters=[(EB, "TCC_HIT_sum", 60.0), (EB, "TCC_REQ_sum", 100.0), (EB, "TCC_MISS_sum", 40.0)])
    bj = str(tmp_path / "b.json")
    bench_json(bj)
    out = str(tmp_path / "hbm.txt")
    res = ps.write_hbm_traffic(str(tmp_path / "f"), str(tmp_path / "w"), str(tmp_path / "t"), str(tmp_path / "cf"),
                               str(tmp_path / "cw"), bj, out, "cmd", us_per_call=100.0)
    assert res["fetch_bytes"] == pytest.approx(2.0 * (2000.0 + 10.0) * 1024)
    assert res["write_bytes"] == pytest.approx(1.0 * (500.0 + 20.0) * 1024)
    assert res["hit"] == pytest.approx(0.6)
    vals = ps.read_summary(out)
    assert float(vals["FETCH_KIB_PER_CALL_SCALED"]) == pytest.approx(4020.0)
    assert float(vals["WRITE_KIB_PER_CALL_SCALED"]) == pytest.approx(520.0)
    assert float(vals["TCC_HIT_RATE"]) == pytest.approx(0.6)


def test_bench_accepts_only_summaries_of_the_same_sources(tmp_path, monkeypatch):
    import bench
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    os.makedirs(tmp_path / "profiles")
    path = tmp_path / "profiles" / "da_spmm_powerlaw_N128_hbm_traffic.txt"
    body = "ALGO = EB+RM+SR\nFETCH_KIB_PER_CALL_SCALED = 1000\nWRITE_KIB_PER_CALL_SCALED = 24\nTCC_HIT_RATE = 0.5\n"
    path.write_text("SOURCE_SHA256 = " + ps.source_hash() + "\n" + body)
    total, hit, note = bench.measured_traffic("powerlaw", 128, "EB+RM+SR")
    assert total == 1024 * 1024 and hit == 0.5 and note.endswith("hbm_traffic.txt")
    assert bench.measured_traffic("powerlaw", 128, "RB+RM+SR")[0] is None          # another algorithm
    path.write_text("SOURCE_SHA256 = 0123\n" + body)
    total, hit, note = bench.measured_traffic("powerlaw", 128, "EB+RM+SR")
    assert total is None and "other kernel sources" in note                        # measured on other sources
    assert bench.measured_traffic("stencil", 32, "RB+RM+SR")[0] is None             # no summary at all
