"""Seeded synthetic inputs for CSR SpMM: sparse matrices A (CSR, int32 indices, fp32 values)
and dense matrices B (row-major fp32).

This module only *draws inputs*.  It contains none of the method's arithmetic (no products,
no reductions over non-zeros, no algorithm selection) so that it can feed both the CPU oracle
and the HIP path without coupling them.  Everything is a pure function of its arguments and
of a numpy ``Generator(PCG64(seed))`` stream.

The paper evaluates on a public sparse-matrix collection that is not available here; the
families below stand in for it and span the input dynamics the paper names as decisive
(Sec. 3.2 row-length dispersion, Sec. 3.3 dense width N, Sec. 3.4 problem size):

  uniform_csr    short rows of similar length, uniform columns
  powerlaw_csr   graph-like: heavy-tailed row lengths, popularity-skewed columns
  stencil27_csr  3-D 27-point stencil: very regular rows, banded columns
  skewed_csr     almost all rows tiny, a handful of enormous rows
  hypersparse_csr  nearly all rows empty, stored rows separated by long runs of empty ones
  sweep_csr      one member j of a 64-matrix family spanning size / density / dispersion
  fig6a_csr      the 5-row 6/2/0/3/1 structure the paper uses to explain its techniques
                 (Sec. 4, Fig. 6(a)); values and columns are not printed there, so they
                 are seeded here
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

__all__ = [
    "CSR", "uniform_csr", "powerlaw_csr", "stencil27_csr", "skewed_csr", "sweep_csr",
    "sweep_params", "fig6a_csr", "lognormal_csr", "rmat_csr", "reversed_edges", "hypersparse_csr",
    "csr_from_lens", "dense", "dense_int", "integer_twin", "config_seed",
]


@dataclass
class CSR:
    """A sparse m x k matrix in CSR form.  rowptr int32[m+1], colind int32[nnz], vals fp32[nnz]."""
    m: int
    k: int
    rowptr: np.ndarray
    colind: np.ndarray
    vals: np.ndarray
    name: str = ""
    seed: int = 0

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    def row_lengths(self) -> np.ndarray:
        return np.diff(self.rowptr.astype(np.int64))


def config_seed(config: int, index: int = 0) -> int:
    """Seed convention: 1000*config + index (index = sweep member for config 5)."""
    return 1000 * config + index


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def _rowptr_from_lens(lens: np.ndarray) -> np.ndarray:
    rp = np.zeros(len(lens) + 1, dtype=np.int64)
    np.cumsum(lens, out=rp[1:])
    if rp[-1] >= 2 ** 31:
        raise ValueError("nnz does not fit int32 row pointers")
    return rp.astype(np.int32)


def _uniform_draw(k: int):
    def draw(rng, rows, n):
        return rng.integers(0, k, size=n, dtype=np.int64)
    return draw


def _distinct_sorted_columns(rng, lens: np.ndarray, k: int, draw) -> np.ndarray:
    """For every row i return lens[i] distinct column ids in ascending order, concatenated.

    ``draw(rng, rows, n)`` returns n candidate columns (int64) for the given row ids; rows
    whose draws collide are topped up with fresh draws until they hold lens[i] distinct ids.
    Rows that still collide after many rounds (only rows nearly as long as k) are finished by
    choosing uniformly among their missing columns.
    """
    lens = np.asarray(lens, dtype=np.int64)
    m = len(lens)
    if np.any(lens > k) or np.any(lens < 0):
        raise ValueError("row length outside [0, k]")
    done = []                       # finished key arrays (key = row*k + col)
    active_rows = np.nonzero(lens > 0)[0]
    keys = np.empty(0, dtype=np.int64)
    deficit = lens[active_rows].copy()
    rounds = 0
    while active_rows.size:
        rep = np.repeat(active_rows, deficit)
        cand = rep * k + draw(rng, rep, rep.size)
        keys = np.unique(np.concatenate([keys, cand]))
        have = np.bincount(np.searchsorted(active_rows, keys // k), minlength=active_rows.size)
        deficit = lens[active_rows] - have
        short = deficit > 0
        if not short.all():
            keep = short[np.searchsorted(active_rows, keys // k)]
            done.append(keys[~keep])
            keys = keys[keep]
            active_rows = active_rows[short]
            deficit = deficit[short]
        rounds += 1
        if rounds >= 48 and active_rows.size:
            # finish the stragglers exactly: pick from the complement of what they hold
            lo = np.searchsorted(keys, active_rows * k)
            hi = np.searchsorted(keys, (active_rows + 1) * k)
            for r, d, a, b in zip(active_rows, deficit, lo, hi):
                held = keys[a:b] % k
                missing = np.setdiff1d(np.arange(k, dtype=np.int64), held, assume_unique=True)
                extra = rng.choice(missing, size=int(d), replace=False)
                done.append(r * k + np.concatenate([held, extra]))
            break
    if not done:
        return np.empty(0, dtype=np.int32)
    allk = np.sort(np.concatenate(done))
    return (allk % k).astype(np.int32)


def csr_from_lens(rng, lens, k: int, draw=None, long_row_frac: float = 1 / 32):
    """Build (rowptr, colind) with the given row lengths and distinct sorted columns.

    Rows longer than long_row_frac*k are drawn one by one without replacement (collisions would
    be frequent); all other rows go through the vectorised draw / de-duplicate / top-up loop.
    """
    lens = np.asarray(lens, dtype=np.int64)
    m = len(lens)
    rowptr = _rowptr_from_lens(lens)
    if draw is None:
        is_long = lens > max(1.0, long_row_frac * k)
        short_lens = np.where(is_long, 0, lens)
        draw_fn = _uniform_draw(k)
    else:
        is_long = np.zeros(m, dtype=bool)
        short_lens = lens
        draw_fn = draw
    cols_short = _distinct_sorted_columns(rng, short_lens, k, draw_fn)
    if not is_long.any():
        return rowptr, cols_short
    colind = np.empty(int(rowptr[-1]), dtype=np.int32)
    # scatter the short rows' columns to their final places
    sp = np.zeros(m + 1, dtype=np.int64)
    np.cumsum(short_lens, out=sp[1:])
    dst = np.repeat(rowptr[:-1].astype(np.int64) - sp[:-1], short_lens) + np.arange(sp[-1])
    colind[dst] = cols_short
    for r in np.nonzero(is_long)[0]:
        c = rng.choice(k, size=int(lens[r]), replace=False)
        c.sort()
        colind[rowptr[r]:rowptr[r + 1]] = c
    return rowptr, colind


def _uniform_vals(rng, n):
    return rng.uniform(-1.0, 1.0, size=n).astype(np.float32)


# ----------------------------------------------------------------------------------------------
# config 1: uniform random
# ----------------------------------------------------------------------------------------------
def uniform_csr(m: int = 4096, k: int = 4096, mean_len: float = 8.0, seed: int = 1000) -> CSR:
    """Row lengths ~ Poisson(mean_len) clipped to [0,k]; columns uniform without replacement,
    sorted; values U(-1,1)."""
    rng = _rng(seed)
    lens = np.minimum(rng.poisson(mean_len, size=m), k)
    rowptr, colind = csr_from_lens(rng, lens, k)
    return CSR(m, k, rowptr, colind, _uniform_vals(rng, colind.size), "uniform", seed)


# ----------------------------------------------------------------------------------------------
# config 2: power-law, graph-like
# ----------------------------------------------------------------------------------------------
def powerlaw_csr(m: int = 262144, k: int | None = None, scale: float = 6.8, max_len: int = 4096,
                 seed: int = 2000) -> CSR:
    """Out-degree with tail exponent 2: len = clip(floor(scale/U), 1, max_len), U ~ U(0,1]
    (P(len >= d) = scale/d; mean ~ 50 at scale 6.8, max_len 4096).  Columns are drawn by
    popularity rank r with P(r) ~ 1/r (r = floor((k+1)^u), u ~ U[0,1)), the rank is mapped to a
    node id through a seeded permutation so that popular rows of B are scattered in memory;
    duplicates inside a row are redrawn.  Values are 1/len (row-normalised adjacency)."""
    k = m if k is None else k
    rng = _rng(seed)
    u = 1.0 - rng.random(m)                       # (0,1]
    lens = np.clip(np.floor(scale / u), 1, min(max_len, k)).astype(np.int64)
    perm = rng.permutation(k).astype(np.int64)
    logk1 = np.log(k + 1.0)

    def draw(rng_, rows, n):
        r = np.floor(np.exp(rng_.random(n) * logk1)).astype(np.int64)   # 1..k
        np.clip(r, 1, k, out=r)
        return perm[r - 1]

    rowptr, colind = csr_from_lens(rng, lens, k, draw=draw)
    vals = np.repeat((1.0 / lens).astype(np.float32), lens)
    return CSR(m, k, rowptr, colind, vals, "powerlaw", seed)


# ----------------------------------------------------------------------------------------------
# config 3: 27-point stencil
# ----------------------------------------------------------------------------------------------
def stencil27_csr(nx: int = 64, ny: int = 128, nz: int = 128, seed: int = 3000,
                  unit_values: bool = False) -> CSR:
    """Non-periodic 27-point stencil on an nx*ny*nz grid.  Row id = x + nx*(y + ny*z) (x fastest).
    Columns ascending.  nnz = (3nx-2)(3ny-2)(3nz-2).  Values U(-1,1) (or all ones)."""
    rng = _rng(seed)
    m = nx * ny * nz
    x = np.arange(m, dtype=np.int64) % nx
    y = (np.arange(m, dtype=np.int64) // nx) % ny
    z = np.arange(m, dtype=np.int64) // (nx * ny)
    offs = [(dx, dy, dz) for dz in (-1, 0, 1) for dy in (-1, 0, 1) for dx in (-1, 0, 1)]
    valid = []
    for dx, dy, dz in offs:
        ok = ((x + dx >= 0) & (x + dx < nx) & (y + dy >= 0) & (y + dy < ny)
              & (z + dz >= 0) & (z + dz < nz))
        valid.append(ok)
    lens = np.zeros(m, dtype=np.int64)
    for ok in valid:
        lens += ok
    rowptr = _rowptr_from_lens(lens)
    colind = np.empty(int(rowptr[-1]), dtype=np.int32)
    pos = rowptr[:-1].astype(np.int64).copy()
    rows = np.arange(m, dtype=np.int64)
    for (dx, dy, dz), ok in zip(offs, valid):        # offsets are in ascending column order
        col = rows + dx + nx * (dy + ny * dz)
        colind[pos[ok]] = col[ok]
        pos += ok
    vals = (np.ones(colind.size, dtype=np.float32) if unit_values
            else _uniform_vals(rng, colind.size))
    return CSR(m, m, rowptr, colind, vals, "stencil27", seed)


# ----------------------------------------------------------------------------------------------
# config 4: skewed rows
# ----------------------------------------------------------------------------------------------
def skewed_csr(m: int = 524288, k: int | None = None, heavy_frac: float = 1e-3,
               light_mean: float = 4.0, heavy_lo: int = 20000, heavy_hi: int = 100000,
               seed: int = 4000) -> CSR:
    """round(heavy_frac*m) rows at seeded positions have length ~ U{heavy_lo..heavy_hi} (clipped
    to k), all others ~ Poisson(light_mean).  Uniform distinct sorted columns, values U(-1,1)."""
    k = m if k is None else k
    rng = _rng(seed)
    lens = np.minimum(rng.poisson(light_mean, size=m), k).astype(np.int64)
    n_heavy = int(round(heavy_frac * m))
    heavy_rows = rng.choice(m, size=n_heavy, replace=False)
    lens[heavy_rows] = np.minimum(rng.integers(heavy_lo, heavy_hi + 1, size=n_heavy), k)
    rowptr, colind = csr_from_lens(rng, lens, k)
    return CSR(m, k, rowptr, colind, _uniform_vals(rng, colind.size), "skewed", seed)


# ----------------------------------------------------------------------------------------------
# config 5: selector sweep family
# ----------------------------------------------------------------------------------------------
def hypersparse_csr(m: int, k: int | None = None, row_frac: float = 0.01, mean_len: float = 100.0,
                    seed: int = 4500) -> CSR:
    """Only round(row_frac*m) rows, at seeded positions, hold entries (length 1 + Poisson(mean_len - 1),
    clipped to k); all other rows are empty, so stored rows are separated by long runs of empty
    ones.  Uniform distinct sorted columns, values U(-1,1)."""
    k = m if k is None else k
    rng = _rng(seed)
    lens = np.zeros(m, dtype=np.int64)
    rows = rng.choice(m, size=max(1, int(round(row_frac * m))), replace=False)
    lens[rows] = np.minimum(1 + rng.poisson(max(mean_len - 1.0, 0.0), size=rows.size), k)
    rowptr, colind = csr_from_lens(rng, lens, k)
    return CSR(m, k, rowptr, colind, _uniform_vals(rng, colind.size), "hypersparse", seed)


def lognormal_csr(m: int, mean_len: float, cv: float, seed: int, k: int | None = None,
                  name: str = "lognormal") -> CSR:
    """Row lengths = clip(round(LogNormal(mu, sigma^2)), 0, k) with sigma^2 = ln(1+cv^2),
    mu = ln(mean_len) - sigma^2/2 (cv = std/mean; cv == 0 gives constant rows).  Uniform
    distinct sorted columns, values U(-1,1)."""
    k = m if k is None else k
    rng = _rng(seed)
    if cv <= 0.0:
        lens = np.full(m, int(round(mean_len)), dtype=np.int64)
    else:
        s2 = np.log1p(cv * cv)
        mu = np.log(mean_len) - 0.5 * s2
        lens = np.rint(rng.lognormal(mu, np.sqrt(s2), size=m)).astype(np.int64)
    lens = np.clip(lens, 0, k)
    rowptr, colind = csr_from_lens(rng, lens, k)
    return CSR(m, k, rowptr, colind, _uniform_vals(rng, colind.size), name, seed)


def sweep_params(j: int, seed_base: int = 5000, max_nnz: int = 2 ** 26):
    """(m, mean_len, cv, seed) of sweep member j: m = round(2^u), u ~ U[12,20]; mean row length
    2^v, v ~ U[1,8]; cv = 0 when j % 8 == 0 else log-uniform in [0.05, 20].  When m*mean_len
    would exceed max_nnz the mean length is lowered to max_nnz/m (keeps one matrix within a
    fraction of device and host memory; the draw itself is unchanged)."""
    seed = seed_base + j
    rng = _rng(seed ^ 0x5EED)
    m = int(round(2.0 ** rng.uniform(12.0, 20.0)))
    mean_len = float(2.0 ** rng.uniform(1.0, 8.0))
    cv = 0.0 if j % 8 == 0 else float(np.exp(rng.uniform(np.log(0.05), np.log(20.0))))
    if m * mean_len > max_nnz:
        mean_len = max_nnz / m
    return m, mean_len, cv, seed


def sweep_csr(j: int, seed_base: int = 5000, max_nnz: int = 2 ** 26) -> CSR:
    m, mean_len, cv, seed = sweep_params(j, seed_base, max_nnz)
    return lognormal_csr(m, mean_len, cv, seed, name=f"sweep{j}")


# ----------------------------------------------------------------------------------------------
# R-MAT graphs for the controlled experiments
# ----------------------------------------------------------------------------------------------
def rmat_csr(scale: int, edge_factor: float = 16.0, a: float = 0.57, b: float = 0.19, c: float = 0.19,
             seed: int = 8000, name: str = "rmat") -> CSR:
    """R-MAT graph on 2^scale nodes (the paper's controlled experiments, Sec. 6.3, synthesise their
    matrices this way; the parameters are not printed there).  Every edge picks one quadrant of the
    adjacency matrix per bit with probabilities (a, b, c, d = 1-a-b-c); duplicate edges are dropped
    and further edges drawn until round(edge_factor * 2^scale) distinct ones exist, so matrices
    that differ only in (a, b, c) have identical size and sparsity.  Values U(-1,1), columns sorted."""
    rng = _rng(seed)
    n = 1 << scale
    target = int(round(edge_factor * n))
    if target > n * n:
        raise ValueError("more edges than matrix entries")
    keys = np.empty(0, dtype=np.int64)
    need = target
    while need > 0:
        e = int(need * 1.15) + 64
        rows = np.zeros(e, dtype=np.int64)
        cols = np.zeros(e, dtype=np.int64)
        for _ in range(scale):
            u = rng.random(e)
            rbit = u >= a + b                       # quadrants c, d: lower half
            cbit = ((u >= a) & (u < a + b)) | (u >= a + b + c)   # quadrants b, d: right half
            rows = rows * 2 + rbit
            cols = cols * 2 + cbit
        new = np.unique(rows * n + cols)
        new = new[~np.isin(new, keys, assume_unique=True)] if keys.size else new
        if new.size > need:
            new = rng.choice(new, size=need, replace=False)
        keys = np.concatenate([keys, new])
        need = target - keys.size
    keys.sort()
    lens = np.bincount(keys // n, minlength=n)
    rowptr = _rowptr_from_lens(lens)
    colind = (keys % n).astype(np.int32)
    return CSR(n, n, rowptr, colind, _uniform_vals(rng, colind.size), name, seed)


def reversed_edges(a: CSR, name: str | None = None) -> CSR:
    """The same graph with every edge reversed (entry (i, j) becomes (j, i), values kept): the matrix
    a GNN's backward pass multiplies with.  For the power-law generator this turns a few popular
    columns into a few very long rows, a much harsher row-length distribution than the original."""
    rows = np.repeat(np.arange(a.m, dtype=np.int64), np.diff(a.rowptr.astype(np.int64)))
    order = np.lexsort((rows, a.colind))                      # by old column, then old row
    lens = np.bincount(a.colind, minlength=a.k)
    return CSR(a.k, a.m, _rowptr_from_lens(lens), rows[order].astype(np.int32), a.vals[order].copy(),
               name or a.name + "_rev", a.seed)


# ----------------------------------------------------------------------------------------------
# the paper's 5-row illustration
# ----------------------------------------------------------------------------------------------
def fig6a_csr(k: int = 8, seed: int = 6) -> CSR:
    """Five rows holding 6/2/0/3/1 non-zeros (Sec. 4, Fig. 6(a)): one row longer than the
    4-wide worker of the illustration, one empty row, one single-entry row.  Columns and values
    are seeded small integers (the text prints neither)."""
    rng = _rng(seed)
    lens = np.array([6, 2, 0, 3, 1], dtype=np.int64)
    rowptr, colind = csr_from_lens(rng, lens, k, long_row_frac=2.0)
    vals = rng.integers(1, 4, size=colind.size).astype(np.float32)
    vals *= rng.choice(np.array([-1.0, 1.0], dtype=np.float32), size=colind.size)
    return CSR(5, k, rowptr, colind, vals, "fig6a", seed)


# ----------------------------------------------------------------------------------------------
# dense operands and integer-valued twins
# ----------------------------------------------------------------------------------------------
def dense(k: int, N: int, dist: str = "uniform", seed: int = 0) -> np.ndarray:
    """Row-major k x N fp32: 'uniform' = U(-1,1), 'normal' = N(0,1)."""
    rng = _rng(seed ^ 0xB0B)
    if dist == "uniform":
        out = rng.random((k, N), dtype=np.float32)
        out *= 2.0
        out -= 1.0
        return out
    if dist == "normal":
        return rng.standard_normal((k, N), dtype=np.float32)
    raise ValueError(dist)


def dense_int(k: int, N: int, seed: int = 0, lo: int = -4, hi: int = 4) -> np.ndarray:
    """Row-major k x N fp32 holding integers in [lo, hi]."""
    rng = _rng(seed ^ 0x1B0B)
    return rng.integers(lo, hi + 1, size=(k, N)).astype(np.float32)


def integer_twin(a: CSR, seed: int | None = None) -> CSR:
    """Same structure, values drawn from {-3,-2,-1,1,2,3}: with dense_int operands every partial
    sum of a row with up to ~1.3e6 entries is an integer below 2^24, hence exact in fp32 in any
    summation order."""
    rng = _rng((a.seed if seed is None else seed) ^ 0x1217)
    mag = rng.integers(1, 4, size=a.colind.size).astype(np.float32)
    sign = rng.integers(0, 2, size=a.colind.size).astype(np.float32) * 2.0 - 1.0
    return CSR(a.m, a.k, a.rowptr, a.colind, mag * sign, a.name + "_int", a.seed)


if __name__ == "__main__":
    # python -m paper_2202_08556_amd.generators <uniform|powerlaw|stencil|skewed> <out.bin>
    # writes the column indices of the benchmark configuration as raw int32 (input of `ceilings file`)
    import sys
    maker = dict(uniform=lambda: uniform_csr(seed=config_seed(1)), powerlaw=lambda: powerlaw_csr(seed=config_seed(2)),
                 stencil=lambda: stencil27_csr(seed=config_seed(3)), skewed=lambda: skewed_csr(seed=config_seed(4)))
    a_ = maker[sys.argv[1]]()
    a_.colind.tofile(sys.argv[2])
    print(f"{sys.argv[1]}: m={a_.m} k={a_.k} nnz={a_.nnz} -> {sys.argv[2]}")
