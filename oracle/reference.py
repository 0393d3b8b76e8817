"""CPU ORACLE -- TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import this module.  It
shares nothing with the HIP path and never imports it.

Contents (each cites the passage of the paper it follows):

  spmm / spmm_rows        the definition Y = A.X in fp64 (Sec. 3.1, Fig. 2(a,b)); thin ctypes
                          marshalling over spmm_oracle.c, which holds the three loops
  dense_view / spmm_ex    the same with X stored row- or column-major with a leading dimension
                          (Sec. 3.3); pinned by explicit index loops on a tiny case
  spmm_transposed         A^T.G from the definition (scatter over A's own entries): the backward
                          pass of the aggregation step of a graph-convolution layer (Sec. 6, GCN)
  csr_transpose           CSR arrays of A^T with ascending indices inside every row
  gcn_layer / gcn_layer_backward   relu(A.(X.W) + b) and its gradients in fp64 (Sec. 6, GCN)
  features                input characteristics of Sec. 5.1, Table 2 (nnz, matrix size, standard
                          deviation of row lengths, N) plus mean / max row length
  conditional_reduction   the conditional prefix-sum network of Sec. 4 (EB+RM+PR, Fig. 6(e)),
                          emulated lane by lane for any worker width
  normalized_performance  the figure of merit of Fig. 1's caption / Sec. 5.1: per input,
                          performance relative to the best algorithm on that input; geometric mean
  tolerance_ratio, bit_mismatches   acceptance tests for an fp32 result against the fp64 oracle

Pins (tests/test_oracle_pins.py): dense fp64 GEMM on tiny inputs, identity / permutation /
diagonal matrices, empty rows, exact integer arithmetic against Python ints, closed forms (row
normalised adjacency times ones; 27-point stencil neighbour counts), linearity and column
independence, entry permutation / splitting, scipy's CSR product, and a literal pure-Python triple
loop.  conditional_reduction is pinned against per-run sums computed by a scalar loop and by the
paper's validity rule on the 6/2/0/3/1 example; normalized_performance against hand-computed
two-input examples.  spmm_transposed / csr_transpose: dense transposes of tiny matrices built by index
loops, scipy's conversion, transposing twice, the structural symmetry of the stencil, and central
differences of <G, A.X>; gcn_layer_backward: central differences of the fp64 forward pass.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spmm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile spmm_oracle.c into liboracle.so with the host C compiler."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, i64 = ctypes.c_void_p, ctypes.c_int64
        lib.oracle_spmm.argtypes = [i64, i64, vp, vp, vp, vp, vp, vp]
        lib.oracle_spmm.restype = None
        lib.oracle_spmm_rows.argtypes = [i64, vp, i64, vp, vp, vp, vp, vp, vp]
        lib.oracle_spmm_rows.restype = None
        lib.oracle_spmm_transposed.argtypes = [i64, i64, i64, vp, vp, vp, vp, vp, vp]
        lib.oracle_spmm_transposed.restype = None
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _prep(rowptr, colind, vals, B):
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colind = np.ascontiguousarray(colind, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    B = np.ascontiguousarray(B, dtype=np.float32)
    if B.ndim != 2:
        raise ValueError("B must be k x N")
    if colind.size and (colind.min() < 0 or colind.max() >= B.shape[0]):
        raise ValueError("column index outside [0, k)")
    if rowptr[0] != 0 or rowptr[-1] != colind.size or np.any(np.diff(rowptr) < 0):
        raise ValueError("malformed rowptr")
    return rowptr, colind, vals, B


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def spmm(rowptr, colind, vals, B, want_abs: bool = True):
    """(C_ref, S_abs) as fp64 m x N arrays: the definition of Sec. 3.1 / Fig. 2 in double precision."""
    rowptr, colind, vals, B = _prep(rowptr, colind, vals, B)
    m, N = rowptr.size - 1, B.shape[1]
    c = np.zeros((m, N), dtype=np.float64)
    s = np.zeros((m, N), dtype=np.float64) if want_abs else None
    if m and N:
        _load().oracle_spmm(m, N, _p(rowptr), _p(colind), _p(vals), _p(B), _p(c), _p(s))
    return c, s


def spmm_rows(rows, rowptr, colind, vals, B, want_abs: bool = True):
    """Rows `rows` of the product only (same loops as spmm); outputs are len(rows) x N."""
    rowptr, colind, vals, B = _prep(rowptr, colind, vals, B)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    if rows.size and (rows.min() < 0 or rows.max() >= rowptr.size - 1):
        raise ValueError("row id out of range")
    N = B.shape[1]
    c = np.zeros((rows.size, N), dtype=np.float64)
    s = np.zeros((rows.size, N), dtype=np.float64) if want_abs else None
    if rows.size and N:
        _load().oracle_spmm_rows(rows.size, _p(rows), N, _p(rowptr), _p(colind), _p(vals), _p(B),
                                 _p(c), _p(s))
    return c, s


def dense_view(buf, rows: int, cols: int, ld: int, col_major: bool):
    """Logical rows x cols matrix stored in a flat buffer with leading dimension ld (Sec. 3.3: X kept
    in row- or column-oriented order): element (r, c) is buf[r*ld + c] (row-major, ld >= cols) or
    buf[r + c*ld] (column-major, ld >= rows).  Returns a view; padding is not part of it."""
    buf = np.asarray(buf).reshape(-1)
    if col_major:
        if ld < rows:
            raise ValueError("ld < rows")
        return buf[: cols * ld].reshape(cols, ld)[:, :rows].T
    if ld < cols:
        raise ValueError("ld < cols")
    return buf[: rows * ld].reshape(rows, ld)[:, :cols]


def spmm_ex(rowptr, colind, vals, b_buf, k: int, N: int, ldb: int, b_col_major: bool, want_abs: bool = True):
    """The definition of Sec. 3.1 with B given in either storage order: decodes the layout, then
    runs the same three loops.  Returns logical m x N arrays (C_ref, S_abs)."""
    return spmm(rowptr, colind, vals, np.ascontiguousarray(dense_view(b_buf, k, N, ldb, b_col_major)), want_abs)


# --------------------------------------------------------------------------------------------
# transposed product, transposed structure and the graph-convolution layer (Sec. 6, GCN)
# --------------------------------------------------------------------------------------------
def spmm_transposed(rowptr, colind, vals, G, k: int, want_abs: bool = True):
    """(D_ref, S_abs) as fp64 k x N arrays with D = A^T.G, where A is m x k and G is m x N: every
    stored entry (i, j) adds vals * G[i, :] to row j.  Gradient of <G, A.X> with respect to X."""
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colind = np.ascontiguousarray(colind, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    G = np.ascontiguousarray(G, dtype=np.float32)
    m = rowptr.size - 1
    if G.ndim != 2 or G.shape[0] != m:
        raise ValueError("G must be m x N")
    if colind.size and (colind.min() < 0 or colind.max() >= k):
        raise ValueError("column index outside [0, k)")
    N = G.shape[1]
    d = np.zeros((k, N), dtype=np.float64)
    s = np.zeros((k, N), dtype=np.float64) if want_abs else None
    if k and N:
        _load().oracle_spmm_transposed(m, k, N, _p(rowptr), _p(colind), _p(vals), _p(G), _p(d), _p(s))
    return d, s


def csr_transpose(rowptr, colind, vals, k: int):
    """CSR arrays (t_rowptr int32[k+1], t_colind int32[nnz], t_vals fp32[nnz]) of A^T for an m x k
    matrix A: row j of A^T lists the entries of column j of A with their row numbers ascending (ties,
    i.e. repeated (i, j) entries, keep their stored order).  A stable sort of the entries by column
    is exactly that, because CSR already stores them row after row."""
    rowptr = np.asarray(rowptr, dtype=np.int64)
    colind = np.asarray(colind, dtype=np.int64)
    vals = np.asarray(vals, dtype=np.float32)
    m = rowptr.size - 1
    row_of_entry = np.repeat(np.arange(m, dtype=np.int64), np.diff(rowptr))
    order = np.argsort(colind, kind="stable")
    t_rowptr = np.zeros(k + 1, dtype=np.int64)
    t_rowptr[1:] = np.cumsum(np.bincount(colind, minlength=k))
    return t_rowptr.astype(np.int32), row_of_entry[order].astype(np.int32), vals[order].copy()


def gcn_layer(rowptr, colind, vals, X, W, bias=None, relu: bool = True):
    """One graph-convolution layer in fp64: Z = A.(X.W) + b, output relu(Z) (or Z).  A is the
    (normalised) adjacency matrix in CSR, X the m x F_in node features, W F_in x F_out.  Returns
    (output, Z)."""
    H = np.asarray(X, dtype=np.float64) @ np.asarray(W, dtype=np.float64)
    rp = np.asarray(rowptr, dtype=np.int64)
    ci = np.asarray(colind, dtype=np.int64)
    va = np.asarray(vals, dtype=np.float64)
    Z = np.zeros((rp.size - 1, H.shape[1]), dtype=np.float64)
    for i in range(rp.size - 1):
        seg = slice(rp[i], rp[i + 1])
        Z[i] = va[seg] @ H[ci[seg]]
    if bias is not None:
        Z = Z + np.asarray(bias, dtype=np.float64)
    return (np.maximum(Z, 0.0) if relu else Z), Z


def gcn_layer_backward(rowptr, colind, vals, X, W, Z, d_out, relu: bool = True):
    """Gradients of sum(d_out * layer output) in fp64: with dZ = d_out masked by Z > 0,
    dH = A^T.dZ, dX = dH.W^T, dW = X^T.dH, db = column sums of dZ.  Returns (dX, dW, db)."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    dZ = np.asarray(d_out, dtype=np.float64) * ((Z > 0.0) if relu else 1.0)
    rp = np.asarray(rowptr, dtype=np.int64)
    ci = np.asarray(colind, dtype=np.int64)
    va = np.asarray(vals, dtype=np.float64)
    dH = np.zeros((X.shape[0], W.shape[1]), dtype=np.float64)
    for i in range(rp.size - 1):
        for p in range(rp[i], rp[i + 1]):
            dH[ci[p]] += va[p] * dZ[i]
    return dH @ W.T, X.T @ dH, dZ.sum(axis=0)


# --------------------------------------------------------------------------------------------
# input characteristics (Sec. 5.1, Table 2)
# --------------------------------------------------------------------------------------------
def features(rowptr, N: int) -> dict:
    """rows (matrix size, read as the number of rows: all workloads are square), nnz, and the
    mean / population standard deviation / maximum of the row lengths, and N."""
    rp = np.asarray(rowptr, dtype=np.int64)
    lens = np.diff(rp)
    m = lens.size
    if m == 0:
        return dict(rows=0, nnz=0, row_nnz_mean=0.0, row_nnz_std=0.0, row_nnz_max=0.0, N=int(N))
    mean = float(lens.sum()) / m
    var = float(((lens.astype(np.float64) - mean) ** 2).sum()) / m
    return dict(rows=int(m), nnz=int(lens.sum()), row_nnz_mean=mean, row_nnz_std=float(np.sqrt(var)),
                row_nnz_max=float(lens.max()), N=int(N))


# --------------------------------------------------------------------------------------------
# conditional reduction (Sec. 4, EB+RM+PR, Fig. 6(e))
# --------------------------------------------------------------------------------------------
def conditional_reduction(partial, index):
    """Emulate the conditional prefix-sum network on one worker of W = len(partial) lanes.

    Every lane holds a partial result and an index flag naming its row; flags are non-decreasing
    from left to right because stored entries are laid out row after row.  In step d = 1, 2, 4, ...
    lane l takes in the value lane l+d held *before* the step, but only if both carry the same
    flag (the datapath is "activated" only then).  Afterwards the value is valid at the leftmost
    lane and at every lane whose flag differs from its left neighbour's: there it equals the sum of
    the whole run of equal flags.  Returns (values after the last step, boolean validity mask).
    """
    v = np.array(partial, dtype=np.float64)
    idx = np.asarray(index)
    W = v.size
    d = 1
    while d < W:
        prev = v.copy()
        for lane in range(W):
            if lane + d < W and idx[lane + d] == idx[lane]:
                v[lane] = prev[lane] + prev[lane + d]
        d *= 2
    valid = np.ones(W, dtype=bool)
    valid[1:] = idx[1:] != idx[:-1]
    return v, valid


# --------------------------------------------------------------------------------------------
# figure of merit of the selector (Fig. 1 caption; Sec. 5.1)
# --------------------------------------------------------------------------------------------
def normalized_performance(times, chosen) -> float:
    """times[i][a] = run time of algorithm a on input i; chosen[i] = algorithm picked for input i.
    Performance is 1/time; each input's figure is perf(chosen)/perf(best on that input); the
    inputs are combined by the geometric mean."""
    t = np.asarray(times, dtype=np.float64)
    ch = np.asarray(chosen, dtype=np.int64)
    best = t.min(axis=1)
    sel = t[np.arange(t.shape[0]), ch]
    return float(np.exp(np.mean(np.log(best / sel))))


# --------------------------------------------------------------------------------------------
# acceptance tests for an fp32 result
# --------------------------------------------------------------------------------------------
REL_TOL = 1e-5
ABS_TOL = 1e-6


def tolerance_ratio(c, c_ref, s_abs) -> float:
    """max over elements of |c - c_ref| / (1e-5 * S_abs + 1e-6); a result passes when <= 1."""
    c = np.asarray(c, dtype=np.float64)
    if c.size == 0:
        return 0.0
    if not np.all(np.isfinite(c)):
        return float("inf")
    return float(np.max(np.abs(c - c_ref) / (REL_TOL * s_abs + ABS_TOL)))


def bit_mismatches(c, c_ref) -> int:
    """Number of elements whose fp32 bit pattern differs from (float)c_ref, after mapping -0 to +0
    (an exact zero sum may carry either sign depending on summation order)."""
    a = np.ascontiguousarray(c, dtype=np.float32) + np.float32(0.0)
    b = np.asarray(c_ref, dtype=np.float64).astype(np.float32) + np.float32(0.0)
    return int(np.count_nonzero(a.view(np.uint32) != b.view(np.uint32)))
