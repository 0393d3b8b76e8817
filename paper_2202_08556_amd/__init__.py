"""DA-SpMM for MI355X (gfx950): CSR sparse x dense matrix multiply over the 8-algorithm space of
the paper's three-loop model (Sec. 3, Table 1) plus data-aware algorithm selection (Sec. 5).

Sub-modules
  generators  seeded synthetic inputs (pure numpy; shared by tests, oracle checks and benchmarks)
  binding     thin ctypes marshalling over the C-ABI library libdaspmm.so (HIP kernels)
  build       compiles the HIP library (and the C oracle used by the tests) in-tree

Importing the package does not load the HIP library; importing ``binding`` does, and raises if
the library has not been built.
"""
__version__ = "0.1.0"
