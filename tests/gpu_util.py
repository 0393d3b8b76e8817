"""Helpers shared by the GPU tests: upload a CSR matrix, run one algorithm id through the C ABI."""
import numpy as np
import torch

from paper_2202_08556_amd import binding as da


class DeviceProblem:
    def __init__(self, a, B):
        dev = torch.device("cuda:0")
        self.a, self.N = a, int(B.shape[1])
        self.rowptr = torch.from_numpy(np.ascontiguousarray(a.rowptr)).to(dev)
        self.colind = torch.from_numpy(np.ascontiguousarray(a.colind)).to(dev)
        self.vals = torch.from_numpy(np.ascontiguousarray(a.vals)).to(dev)
        self.B = torch.from_numpy(np.ascontiguousarray(B)).to(dev)

    def run(self, algo, fill=float("nan")):
        """C is pre-filled with NaN so that any element the library fails to overwrite shows."""
        C = torch.full((self.a.m, self.N), fill, device=self.B.device, dtype=torch.float32)
        da.da_spmm(self.a.m, self.a.k, self.N, self.rowptr, self.colind, self.vals, self.B, C, algo)
        torch.cuda.synchronize()
        return C.cpu().numpy()
