"""Thin Python binding over the C ABI of libdaspmm.so (include/da_spmm.h).

Argument marshalling only: every step of the SpMM path runs in the HIP kernels of the library.
PyTorch is used for device memory and streams.  Importing this module loads the library and
raises ImportError if it has not been built (python -m paper_2202_08556_amd.build); there is
no CPU or PyTorch fallback.
"""
from __future__ import annotations

import ctypes
import os

import torch  # loads the HIP runtime the library links against

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdaspmm.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2202_08556_amd.build`")
_lib = ctypes.CDLL(_LIB_PATH)

DA_OK, DA_ERR_INVALID_ARG, DA_ERR_BAD_ALGO, DA_ERR_UNSUPPORTED, DA_ERR_HIP = range(5)
(DA_RB_RM_SR, DA_RB_RM_PR, DA_RB_CM_SR, DA_RB_CM_PR,
 DA_EB_RM_SR, DA_EB_RM_PR, DA_EB_CM_SR, DA_EB_CM_PR) = range(8)
DA_NUM_ALGOS = 8
DA_ROW_MAJOR, DA_COL_MAJOR = 0, 1
EXPORTS = ("da_spmm", "da_spmm_ex", "da_spmm_select", "da_spmm_features", "da_csr_transpose_workspace",
           "da_csr_transpose", "da_csr_transpose_noalloc", "da_csr_validate", "da_spmm_prepare", "da_spmm_release",
           "da_eb_schedule_workspace", "da_eb_schedule", "da_spmm_algo_name", "da_spmm_last_error")


class da_features(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("row_nnz_mean", ctypes.c_double), ("row_nnz_std", ctypes.c_double),
                ("row_nnz_max", ctypes.c_double), ("N", ctypes.c_int64)]


_vp, _i64 = ctypes.c_void_p, ctypes.c_int64
_lib.da_spmm.argtypes = [_i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, ctypes.c_int, _vp]
_lib.da_spmm.restype = ctypes.c_int
_lib.da_spmm_ex.argtypes = [_i64, _i64, _i64, _vp, _vp, _vp, _vp, _i64, ctypes.c_int, _vp, _i64, ctypes.c_int,
                            ctypes.c_int, _vp]
_lib.da_spmm_ex.restype = ctypes.c_int
_lib.da_spmm_select.argtypes = [ctypes.POINTER(da_features)]
_lib.da_spmm_select.restype = ctypes.c_int
_lib.da_spmm_features.argtypes = [_i64, _i64, _vp, _vp, ctypes.POINTER(da_features)]
_lib.da_spmm_features.restype = ctypes.c_int
_lib.da_csr_transpose_workspace.argtypes = [_i64, _i64, _i64, ctypes.POINTER(ctypes.c_size_t)]
_lib.da_csr_transpose_workspace.restype = ctypes.c_int
_lib.da_csr_transpose.argtypes = [_i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.da_csr_transpose.restype = ctypes.c_int
_lib.da_csr_transpose_noalloc.argtypes = [_i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.da_csr_transpose_noalloc.restype = ctypes.c_int
_lib.da_csr_validate.argtypes = [_i64, _i64, _i64, _vp, _vp, _vp]
_lib.da_csr_validate.restype = ctypes.c_int
_lib.da_spmm_prepare.argtypes = [_i64, _i64, _i64, _vp, _vp, _vp]
_lib.da_spmm_prepare.restype = ctypes.c_int
_lib.da_spmm_release.argtypes = [_vp]
_lib.da_spmm_release.restype = ctypes.c_int
_lib.da_eb_schedule_workspace.argtypes = [_i64, _i64, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
_lib.da_eb_schedule_workspace.restype = ctypes.c_int
_lib.da_eb_schedule.argtypes = [_i64, _i64, _i64, _vp, _vp, ctypes.c_int, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.da_eb_schedule.restype = ctypes.c_int
_lib.da_spmm_algo_name.argtypes = [ctypes.c_int]
_lib.da_spmm_algo_name.restype = ctypes.c_char_p
_lib.da_spmm_last_error.argtypes = []
_lib.da_spmm_last_error.restype = ctypes.c_char_p


class DaSpmmError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"da_spmm status {status}: {message}")
        self.status = status


def _ptr(x):
    """Device address of a torch tensor, or an int / None passed through."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def da_spmm_last_error() -> str:
    return _lib.da_spmm_last_error().decode()


def da_spmm_status(m, k, N, rowptr, colind, vals, B, C, algo, stream=None) -> int:
    """Raw call: returns the da_status instead of raising."""
    return int(_lib.da_spmm(int(m), int(k), int(N), _ptr(rowptr), _ptr(colind), _ptr(vals),
                            _ptr(B), _ptr(C), int(algo), _stream(stream)))


def da_spmm(m, k, N, rowptr, colind, vals, B, C, algo, stream=None) -> None:
    """C = A.B on the device; arguments as in include/da_spmm.h (torch CUDA tensors or addresses)."""
    st = da_spmm_status(m, k, N, rowptr, colind, vals, B, C, algo, stream)
    if st != DA_OK:
        raise DaSpmmError(st, da_spmm_last_error())


def da_spmm_ex_status(m, k, N, rowptr, colind, vals, B, ldb, layout_b, C, ldc, layout_c, algo, stream=None) -> int:
    return int(_lib.da_spmm_ex(int(m), int(k), int(N), _ptr(rowptr), _ptr(colind), _ptr(vals), _ptr(B), int(ldb),
                               int(layout_b), _ptr(C), int(ldc), int(layout_c), int(algo), _stream(stream)))


def da_spmm_ex(m, k, N, rowptr, colind, vals, B, ldb, layout_b, C, ldc, layout_c, algo, stream=None) -> None:
    """C = A.B with explicit storage order (DA_ROW_MAJOR / DA_COL_MAJOR) and leading dimensions."""
    st = da_spmm_ex_status(m, k, N, rowptr, colind, vals, B, ldb, layout_b, C, ldc, layout_c, algo, stream)
    if st != DA_OK:
        raise DaSpmmError(st, da_spmm_last_error())


class PreparedSpmm:
    """The same call with its arguments marshalled once: `run = PreparedSpmm(m, k, N, rowptr, colind,
    vals, B, C, stream); run(algo)`.  Saves the per-call conversion cost (about 4 us in CPython),
    which matters when the product itself takes a few microseconds.  The tensors must stay alive and
    the stream is the one current when the object was made (or the one given)."""

    def __init__(self, m, k, N, rowptr, colind, vals, B, C, stream=None, ldb=None, layout_b=DA_ROW_MAJOR,
                 ldc=None, layout_c=DA_ROW_MAJOR):
        self._keep = (rowptr, colind, vals, B, C)
        ldb = (N if layout_b == DA_ROW_MAJOR else k) if ldb is None else ldb
        ldc = (N if layout_c == DA_ROW_MAJOR else m) if ldc is None else ldc
        self._args = (_i64(int(m)), _i64(int(k)), _i64(int(N)), _vp(_ptr(rowptr)), _vp(_ptr(colind)),
                      _vp(_ptr(vals)), _vp(_ptr(B)), _i64(int(ldb)), ctypes.c_int(int(layout_b)),
                      _vp(_ptr(C)), _i64(int(ldc)), ctypes.c_int(int(layout_c)))
        self._stream = _vp(_stream(stream))
        self._fn = _lib.da_spmm_ex

    def __call__(self, algo: int) -> None:
        st = self._fn(*self._args, algo, self._stream)
        if st != DA_OK:
            raise DaSpmmError(st, da_spmm_last_error())


def _to_struct(f) -> da_features:
    if isinstance(f, da_features):
        return f
    return da_features(int(f["rows"]), int(f["nnz"]), float(f["row_nnz_mean"]),
                       float(f["row_nnz_std"]), float(f["row_nnz_max"]), int(f["N"]))


def da_spmm_select(f) -> int:
    """Algorithm id for the given features (dict with the fields of da_features, or the struct)."""
    if f is None:
        r = int(_lib.da_spmm_select(None))
    else:
        s = _to_struct(f)
        r = int(_lib.da_spmm_select(ctypes.byref(s)))
    if r < 0:
        raise DaSpmmError(-r, "da_spmm_select: invalid features")
    return r


def da_spmm_features(m, N, rowptr, stream=None) -> dict:
    out = da_features()
    st = int(_lib.da_spmm_features(int(m), int(N), _ptr(rowptr), _stream(stream), ctypes.byref(out)))
    if st != DA_OK:
        raise DaSpmmError(st, da_spmm_last_error())
    return {n: getattr(out, n) for n, _ in da_features._fields_}


def da_csr_transpose_workspace(m, k, nnz) -> int:
    """Bytes of device workspace da_csr_transpose needs."""
    out = ctypes.c_size_t(0)
    st = int(_lib.da_csr_transpose_workspace(int(m), int(k), int(nnz), ctypes.byref(out)))
    if st != DA_OK:
        raise DaSpmmError(st, da_spmm_last_error())
    return int(out.value)


def da_csr_transpose_status(m, k, nnz, rowptr, colind, vals, t_rowptr, t_colind, t_vals, workspace,
                            workspace_bytes, stream=None) -> int:
    return int(_lib.da_csr_transpose(int(m), int(k), int(nnz), _ptr(rowptr), _ptr(colind), _ptr(vals),
                                     _ptr(t_rowptr), _ptr(t_colind), _ptr(t_vals), _ptr(workspace),
                                     int(workspace_bytes), _stream(stream)))


def da_csr_transpose(m, k, nnz, rowptr, colind, vals, t_rowptr, t_colind, t_vals, workspace, workspace_bytes,
                     stream=None) -> None:
    """CSR arrays of A^T on the device; arguments as in include/da_spmm.h."""
    st = da_csr_transpose_status(m, k, nnz, rowptr, colind, vals, t_rowptr, t_colind, t_vals, workspace,
                                 workspace_bytes, stream)
    if st != DA_OK:
        raise DaSpmmError(st, da_spmm_last_error())


DA_NOALLOC_SCRATCH_BYTES = 32 << 20


def da_csr_transpose_noalloc_status(m, k, nnz, rowptr, colind, vals, t_rowptr, t_colind, t_vals, stream=None) -> int:
    return int(_lib.da_csr_transpose_noalloc(int(m), int(k), int(nnz), _ptr(rowptr), _ptr(colind), _ptr(vals),
                                             _ptr(t_rowptr), _ptr(t_colind), _ptr(t_vals), _stream(stream)))


def da_csr_transpose_noalloc(m, k, nnz, rowptr, colind, vals, t_rowptr, t_colind, t_vals, stream=None) -> None:
    """da_csr_transpose on the library's static scratch: no workspace, no allocation (see include/da_spmm.h)."""
    _check(da_csr_transpose_noalloc_status(m, k, nnz, rowptr, colind, vals, t_rowptr, t_colind, t_vals, stream))


def da_csr_validate_status(m, k, nnz, rowptr, colind, stream=None) -> int:
    return int(_lib.da_csr_validate(int(m), int(k), int(nnz), _ptr(rowptr), _ptr(colind), _stream(stream)))


def da_csr_validate(m, k, nnz, rowptr, colind, stream=None) -> None:
    """Raise DaSpmmError unless the CSR arrays are well formed (nnz = -1: do not compare rowptr[m])."""
    st = da_csr_validate_status(m, k, nnz, rowptr, colind, stream)
    if st != DA_OK:
        raise DaSpmmError(st, da_spmm_last_error())


def _check(st: int) -> None:
    if st != DA_OK:
        raise DaSpmmError(st, da_spmm_last_error())


def da_spmm_prepare(m, k, nnz, rowptr, colind, stream=None) -> None:
    """Build and keep the EB chunk orders of this matrix (see include/da_spmm.h)."""
    _check(int(_lib.da_spmm_prepare(int(m), int(k), int(nnz), _ptr(rowptr), _ptr(colind), _stream(stream))))


def da_spmm_release(rowptr=None) -> None:
    """Drop the prepared orders of one matrix (or of all, with None)."""
    _check(int(_lib.da_spmm_release(_ptr(rowptr))))


def da_eb_schedule_workspace(k, nnz, unit) -> int:
    out = ctypes.c_size_t(0)
    _check(int(_lib.da_eb_schedule_workspace(int(k), int(nnz), int(unit), ctypes.byref(out))))
    return int(out.value)


def da_eb_schedule_status(m, k, nnz, rowptr, colind, unit, order, first_segment, workspace, workspace_bytes,
                          stream=None) -> int:
    return int(_lib.da_eb_schedule(int(m), int(k), int(nnz), _ptr(rowptr), _ptr(colind), int(unit), _ptr(order),
                                   _ptr(first_segment), _ptr(workspace), int(workspace_bytes), _stream(stream)))


def da_eb_schedule(m, k, nnz, rowptr, colind, unit, order, first_segment, workspace, workspace_bytes,
                   stream=None) -> None:
    _check(da_eb_schedule_status(m, k, nnz, rowptr, colind, unit, order, first_segment, workspace, workspace_bytes,
                                 stream))


def da_spmm_algo_name(algo: int):
    s = _lib.da_spmm_algo_name(int(algo))
    return s.decode() if s is not None else None


ALGO_NAMES = [da_spmm_algo_name(a) for a in range(DA_NUM_ALGOS)]
