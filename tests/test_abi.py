"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, rejects bad arguments before touching the device, and the selector is a total,
deterministic function."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2202_08556_amd", "libdaspmm.so")

if not os.path.exists(LIB):
    from paper_2202_08556_amd import build as _b
    _b.build_hip()

from paper_2202_08556_amd import binding as da  # noqa: E402


def declared_functions():
    text = open(os.path.join(ROOT, "include", "da_spmm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(da_(?:spmm|csr|eb)\w*)\s*\(", text)))


def test_header_symbols_are_exported():
    names = declared_functions()
    assert set(names) == set(da.EXPORTS)
    lib = ctypes.CDLL(LIB)
    for n in names:
        assert getattr(lib, n) is not None


def test_algo_names_follow_table1_order():
    assert da.ALGO_NAMES == ["RB+RM+SR", "RB+RM+PR", "RB+CM+SR", "RB+CM+PR",
                             "EB+RM+SR", "EB+RM+PR", "EB+CM+SR", "EB+CM+PR"]
    assert da.da_spmm_algo_name(8) is None and da.da_spmm_algo_name(-1) is None


def test_argument_errors_without_device_work():
    f = da.da_spmm_status
    assert f(-1, 4, 4, 0, 0, 0, 0, 0, 0, stream=0) == da.DA_ERR_INVALID_ARG
    assert "negative" in da.da_spmm_last_error()
    assert f(4, 4, -2, 0, 0, 0, 0, 0, 0, stream=0) == da.DA_ERR_INVALID_ARG
    assert f(2 ** 31, 4, 4, 0, 0, 0, 0, 0, 0, stream=0) == da.DA_ERR_INVALID_ARG
    assert f(4, 4, 4, 0, 0, 0, 0, 0, 8, stream=0) == da.DA_ERR_BAD_ALGO
    assert f(4, 4, 4, 0, 0, 0, 0, 0, -1, stream=0) == da.DA_ERR_BAD_ALGO
    assert f(4, 4, 4, None, None, None, None, None, 0, stream=0) == da.DA_ERR_INVALID_ARG   # null pointers
    assert f(0, 4, 4, None, None, None, None, None, 3, stream=0) == da.DA_OK               # m == 0: no-op
    assert f(4, 4, 0, None, None, None, None, None, 5, stream=0) == da.DA_OK               # N == 0: no-op
    with pytest.raises(da.DaSpmmError):
        da.da_spmm(4, 4, 4, None, None, None, None, None, 0, stream=0)


def test_transpose_argument_errors_without_device_work():
    assert da.da_csr_transpose_workspace(10, 10, 0) >= 0
    big = da.da_csr_transpose_workspace(1 << 20, 1 << 20, 1 << 24)
    assert big >= 4 * 4 * (1 << 24) and big % 256 == 0            # two key and two payload buffers at least
    with pytest.raises(da.DaSpmmError):
        da.da_csr_transpose_workspace(-1, 10, 5)
    with pytest.raises(da.DaSpmmError):
        da.da_csr_transpose_workspace(10, 10, 1 << 31)
    f = da.da_csr_transpose_status
    assert f(-1, 4, 4, 0, 0, 0, 0, 0, 0, 0, 0, stream=0) == da.DA_ERR_INVALID_ARG
    assert f(4, 4, 4, 1, 1, 1, None, 1, 1, 1, 1 << 20, stream=0) == da.DA_ERR_INVALID_ARG     # null t_rowptr
    assert f(4, 4, 4, 1, None, 1, 1, 1, 1, 1, 1 << 20, stream=0) == da.DA_ERR_INVALID_ARG     # null colind
    assert f(0, 4, 4, 1, 1, 1, 1, 1, 1, 1, 1 << 20, stream=0) == da.DA_ERR_INVALID_ARG        # entries without rows
    assert f(4, 4, 4, 256, 256, 256, 256, 256, 256, 256, 16, stream=0) == da.DA_ERR_INVALID_ARG   # workspace too small
    assert "workspace" in da.da_spmm_last_error()


def test_validate_argument_errors_without_device_work():
    f = da.da_csr_validate_status
    assert f(-1, 4, 0, 0, 0, stream=0) == da.DA_ERR_INVALID_ARG
    assert f(4, 4, -2, 0, 0, stream=0) == da.DA_ERR_INVALID_ARG
    assert f(2 ** 31, 4, 0, 0, 0, stream=0) == da.DA_ERR_INVALID_ARG
    assert f(0, 4, 0, None, None, stream=0) == da.DA_OK
    assert f(0, 4, 3, None, None, stream=0) == da.DA_ERR_INVALID_ARG
    assert f(4, 4, 3, None, None, stream=0) == da.DA_ERR_INVALID_ARG          # null rowptr
    with pytest.raises(da.DaSpmmError):
        da.da_csr_validate(4, 4, 3, None, None, stream=0)


def test_ex_argument_errors_without_device_work():
    f = da.da_spmm_ex_status
    R, Cm = da.DA_ROW_MAJOR, da.DA_COL_MAJOR
    assert f(4, 6, 8, 0, 0, 0, 0, 8, 2, 0, 8, R, 0, stream=0) == da.DA_ERR_INVALID_ARG      # unknown layout
    assert f(4, 6, 8, 0, 0, 0, 0, 7, R, 0, 8, R, 0, stream=0) == da.DA_ERR_INVALID_ARG      # ldb < N
    assert f(4, 6, 8, 0, 0, 0, 0, 5, Cm, 0, 8, R, 0, stream=0) == da.DA_ERR_INVALID_ARG     # ldb < k
    assert f(4, 6, 8, 0, 0, 0, 0, 8, R, 0, 3, Cm, 0, stream=0) == da.DA_ERR_INVALID_ARG     # ldc < m
    assert "leading dimension" in da.da_spmm_last_error()
    assert f(0, 6, 8, None, None, None, None, 8, R, None, 8, R, 0, stream=0) == da.DA_OK
    assert f(4, 6, 8, None, None, None, None, 8, R, None, 8, R, 9, stream=0) == da.DA_ERR_BAD_ALGO


def feats(rows, mean, cv, mx, N):
    return dict(rows=rows, nnz=int(rows * mean), row_nnz_mean=mean, row_nnz_std=cv * mean,
                row_nnz_max=mx, N=N)


def test_selector_total_and_deterministic():
    rng = np.random.Generator(np.random.PCG64(1))
    for _ in range(2000):
        rows = int(2 ** rng.uniform(0, 24))
        mean = float(2 ** rng.uniform(-2, 10))
        f = feats(rows, mean, float(rng.uniform(0, 30)), mean * float(rng.uniform(1, 2000)),
                  int(2 ** rng.uniform(0, 10)))
        a = da.da_spmm_select(f)
        assert 0 <= a < 8 and a == da.da_spmm_select(f)
    assert 0 <= da.da_spmm_select(feats(0, 0.0, 0.0, 0.0, 0)) < 8          # degenerate but valid


def test_selector_rejects_bad_features():
    for bad in (dict(rows=-1), dict(nnz=-5), dict(N=-1), dict(row_nnz_mean=float("nan")),
                dict(row_nnz_std=-1.0), dict(row_nnz_max=float("inf"))):
        f = feats(100, 4.0, 0.5, 9.0, 8)
        f.update(bad)
        with pytest.raises(da.DaSpmmError):
            da.da_spmm_select(f)
    with pytest.raises(da.DaSpmmError):
        da.da_spmm_select(None)


def test_features_argument_errors():
    out = da.da_features()
    assert da._lib.da_spmm_features(-1, 8, None, None, ctypes.byref(out)) == da.DA_ERR_INVALID_ARG
    assert da._lib.da_spmm_features(4, 8, None, None, None) == da.DA_ERR_INVALID_ARG
    assert da._lib.da_spmm_features(0, 8, None, None, ctypes.byref(out)) == da.DA_OK
    assert out.rows == 0 and out.nnz == 0 and out.N == 8
