"""Graph-convolution layer on top of the C ABI: the application of the paper's Sec. 6, where the
data-aware SpMM replaces the framework's aggregation kernel inside GCN layers.

    Z = A . (X . W) + b,   out = relu(Z)

A is the (normalised) adjacency matrix in CSR, X the node features.  The aggregation A.H runs in
da_spmm with the algorithm the selector picks for (A, feature length); its backward pass, the
gradient A^T.dZ, runs in da_spmm on the CSR arrays of A^T, which da_csr_transpose builds once per
graph, with the algorithm the selector picks for (A^T, feature length).  The dense product X.W is
a plain library GEMM (torch.matmul).  This module only allocates tensors and marshals arguments;
there is no fallback when the HIP library is missing (importing ``binding`` raises).
"""
from __future__ import annotations

import torch

from . import binding as da


class SparseGraph:
    """CSR matrix A (m x k) resident on the device, with its selector features, the algorithm
    chosen per feature length, and (built on first use) A^T.

    The first product prepares the matrix (da_spmm_prepare: EB chunk order and row hints).  The
    library keeps the plans of the 16 most recently prepared matrices; a program that holds more
    graphs than that (a graph and its transpose count as two) loses the oldest plans silently, which
    costs the EB algorithms their chunk order (speed), never the result."""

    def __init__(self, m: int, k: int, rowptr: torch.Tensor, colind: torch.Tensor, vals: torch.Tensor):
        if rowptr.dtype != torch.int32 or colind.dtype != torch.int32 or vals.dtype != torch.float32:
            raise TypeError("rowptr / colind must be int32 and vals float32")
        if not (rowptr.is_cuda and colind.is_cuda and vals.is_cuda):
            raise ValueError("CSR arrays must live on the GPU")
        if rowptr.numel() != m + 1 or colind.numel() != vals.numel():
            raise ValueError("CSR array sizes do not match")
        self.m, self.k, self.nnz = int(m), int(k), int(colind.numel())
        self.rowptr, self.colind, self.vals = rowptr.contiguous(), colind.contiguous(), vals.contiguous()
        self._features = None
        self._algo = {}
        self._t = None
        self._prepared = False

    @classmethod
    def from_numpy(cls, a, device="cuda:0") -> "SparseGraph":
        """From an object with fields m, k, rowptr, colind, vals (e.g. generators.CSR)."""
        dev = torch.device(device)
        return cls(a.m, a.k, torch.from_numpy(a.rowptr).to(dev), torch.from_numpy(a.colind).to(dev),
                   torch.from_numpy(a.vals).to(dev))

    def __del__(self):
        if getattr(self, "_prepared", False):
            try:
                da.da_spmm_release(self.rowptr)
            except Exception:
                pass

    def features(self, N: int) -> dict:
        if self._features is None:
            self._features = da.da_spmm_features(self.m, 1, self.rowptr)     # one device reduction per graph
        f = dict(self._features)
        f["N"] = int(N)
        return f

    def algo_for(self, N: int) -> int:
        """Algorithm id the selector picks for this matrix and feature length (cached)."""
        if N not in self._algo:
            self._algo[N] = da.da_spmm_select(self.features(N))
        return self._algo[N]

    def transposed(self) -> "SparseGraph":
        """A^T as a SparseGraph (k x m); built once by da_csr_transpose."""
        if self._t is None:
            dev = self.rowptr.device
            t_rowptr = torch.empty(self.k + 1, dtype=torch.int32, device=dev)
            t_colind = torch.empty(self.nnz, dtype=torch.int32, device=dev)
            t_vals = torch.empty(self.nnz, dtype=torch.float32, device=dev)
            nbytes = da.da_csr_transpose_workspace(self.m, self.k, self.nnz)
            # scratch of the call; torch allocations are 512-byte aligned and the caching allocator keeps
            # the block alive for work already queued on this stream
            ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
            da.da_csr_transpose(self.m, self.k, self.nnz, self.rowptr, self.colind, self.vals,
                                t_rowptr, t_colind, t_vals, ws, nbytes)
            self._t = SparseGraph(self.k, self.m, t_rowptr, t_colind, t_vals)
            self._t._t = self
        return self._t

    def spmm(self, X: torch.Tensor, algo: int | None = None) -> torch.Tensor:
        """A . X for a row-major fp32 k x N tensor on the same device; returns a new m x N tensor."""
        if X.dtype != torch.float32 or X.dim() != 2 or X.shape[0] != self.k:
            raise ValueError("X must be a float32 k x N tensor")
        X = X.contiguous()
        N = int(X.shape[1])
        if not self._prepared:                      # one-off: chunk order for the EB algorithms
            da.da_spmm_prepare(self.m, self.k, self.nnz, self.rowptr, self.colind)
            self._prepared = True
        C = torch.empty((self.m, N), dtype=torch.float32, device=X.device)
        da.da_spmm(self.m, self.k, N, self.rowptr, self.colind, self.vals, X, C,
                   self.algo_for(N) if algo is None else algo)
        return C


class _Aggregate(torch.autograd.Function):
    @staticmethod
    def forward(ctx, X, graph):
        ctx.graph = graph
        return graph.spmm(X)

    @staticmethod
    def backward(ctx, dY):
        return ctx.graph.transposed().spmm(dY), None


def aggregate(graph: SparseGraph, X: torch.Tensor) -> torch.Tensor:
    """A . X with gradient A^T . dY with respect to X (A itself is a constant of the graph)."""
    return _Aggregate.apply(X, graph)


class GraphConv(torch.nn.Module):
    """relu(A . (X . W) + b): one GCN layer (Sec. 6) whose aggregation is da_spmm."""

    def __init__(self, in_features: int, out_features: int, bias: bool = True, relu: bool = True):
        super().__init__()
        self.weight = torch.nn.Parameter(torch.empty(in_features, out_features))
        self.bias = torch.nn.Parameter(torch.zeros(out_features)) if bias else None
        self.relu = relu
        torch.nn.init.xavier_uniform_(self.weight)

    def forward(self, graph: SparseGraph, X: torch.Tensor) -> torch.Tensor:
        Z = aggregate(graph, X @ self.weight)
        if self.bias is not None:
            Z = Z + self.bias
        return torch.relu(Z) if self.relu else Z
