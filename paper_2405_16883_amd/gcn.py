"""One graph-convolution layer  H' = act(A_hat H W + b)  on top of the C ABI (paper, Section 5.1).

The dense product is left to the dense library (torch.mm), as the paper leaves dense work to PyTorch; the
neighbourhood aggregation, the bias and the activation run in scorch_spmm_csr_planned_epilogue.  The order of the two
products is chosen by width: the aggregation costs 2*nnz*n flops and gathers n floats per stored entry, so it is done
at the narrower of the two feature widths:

    n_out <= n_in :  H' = act(A_hat (H W) + b)      dense product first, epilogue fused into the aggregation
    n_out >  n_in :  H' = act((A_hat H) W + b)      aggregation first, bias and activation applied by the dense side

Orchestration only: no sparse arithmetic happens in this file.
"""
from __future__ import annotations

from typing import Dict, Optional

import torch

from . import binding as _b


class GcnLayer:
    """Holds the normalised adjacency (CSR, device tensors) and one plan per feature width it has been used with."""

    def __init__(self, m: int, rowptr: torch.Tensor, colidx: torch.Tensor, vals: torch.Tensor, nnz: int):
        self.m, self.nnz = int(m), int(nnz)
        self.rowptr, self.colidx, self.vals = rowptr, colidx, vals
        self._plans: Dict[int, _b.SpmmPlan] = {}

    def _plan(self, n: int) -> _b.SpmmPlan:
        if n not in self._plans:
            self._plans[n] = _b.scorch_spmm_plan(self.m, self.m, n, self.rowptr, self.nnz, colidx=self.colidx)
        return self._plans[n]

    @staticmethod
    def aggregates_first(n_in: int, n_out: int) -> bool:
        return n_out > n_in

    def forward(self, H: torch.Tensor, W: torch.Tensor, bias: Optional[torch.Tensor] = None, relu: bool = True,
                stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
        n_in, n_out = int(W.shape[0]), int(W.shape[1])
        if H.shape != (self.m, n_in):
            raise ValueError(f"H must be {self.m} x {n_in}")
        act = _b.ACT_RELU if relu else _b.ACT_IDENTITY
        if not self.aggregates_first(n_in, n_out):
            Z = torch.mm(H, W)
            out = torch.empty((self.m, n_out), dtype=torch.float32, device=H.device)
            _b.scorch_spmm_csr_planned_epilogue(self._plan(n_out), self.rowptr, self.colidx, self.vals, Z, bias, act, out,
                                                stream=stream)
            return out
        Y = torch.empty((self.m, n_in), dtype=torch.float32, device=H.device)
        _b.scorch_spmm_csr_planned(self._plan(n_in), self.rowptr, self.colidx, self.vals, H, Y, stream=stream)
        # Here the dense product comes last, so bias and activation are the epilogue of a DENSE operation: they stay
        # with the dense library (addmm adds the bias inside the product, relu_ runs on its result), exactly as the
        # paper hands dense work to PyTorch.  Nothing sparse is computed in Python.
        out = torch.mm(Y, W) if bias is None else torch.addmm(bias, Y, W)
        return torch.relu_(out) if relu else out

    def close(self) -> None:
        for p in self._plans.values():
            p.destroy()
        self._plans.clear()
