"""Helpers for the GPU parity tests: upload a problem, run the HIP path through the C ABI, compare with the oracle."""
from __future__ import annotations

import os
from contextlib import contextmanager

import numpy as np
import torch

import paper_2405_16883_amd as sp
from oracle import spmm_csr_oracle

RTOL_T = 1e-5  # |C - C_ref| <= RTOL_T * (|A|.|B|) + ATOL per element
ATOL = 1e-7
SENTINEL = -12345.5


@contextmanager
def tuning(spec: str | None):
    old = os.environ.get("SCORCH_SPMM_TUNE")
    if spec is None:
        os.environ.pop("SCORCH_SPMM_TUNE", None)
    else:
        os.environ["SCORCH_SPMM_TUNE"] = spec
    try:
        yield
    finally:
        if old is None:
            os.environ.pop("SCORCH_SPMM_TUNE", None)
        else:
            os.environ["SCORCH_SPMM_TUNE"] = old


class DeviceProblem:
    def __init__(self, p, ldc=None, dev="cuda:0"):
        self.p = p
        self.dev = torch.device(dev)
        self.rowptr = torch.from_numpy(p.rowptr).to(self.dev)
        self.colidx = torch.from_numpy(p.colidx).to(self.dev) if p.nnz else torch.zeros(0, dtype=torch.int32, device=self.dev)
        self.vals = torch.from_numpy(p.vals).to(self.dev) if p.nnz else torch.zeros(0, dtype=torch.float32, device=self.dev)
        self.Bfull = torch.from_numpy(np.ascontiguousarray(p.B)).to(self.dev)
        self.B = self.Bfull[:, :p.n] if p.n else self.Bfull
        self.ldc = ldc if ldc is not None else p.n
        self.Cfull = torch.full((max(p.m, 1), max(self.ldc, 1)), SENTINEL, dtype=torch.float32, device=self.dev)
        self.C = self.Cfull[:p.m, :p.n]

    def reset_C(self):
        self.Cfull.fill_(SENTINEL)

    def run_natural(self):
        p = self.p
        self.reset_C()
        sp.scorch_spmm_csr(p.m, p.k, p.n, self.rowptr, self.colidx, self.vals, self._B_arg(), self._C_arg())
        torch.cuda.synchronize()
        return self.Cfull.cpu().numpy()

    def make_plan(self, with_colidx=True):
        p = self.p
        return sp.scorch_spmm_plan(p.m, p.k, p.n, self.rowptr, p.nnz, colidx=self.colidx if with_colidx else None)

    def run_planned(self, plan):
        self.reset_C()
        sp.scorch_spmm_csr_planned(plan, self.rowptr, self.colidx, self.vals, self._B_arg(), self._C_arg())
        torch.cuda.synchronize()
        return self.Cfull.cpu().numpy()

    def _B_arg(self):
        # a view with the real row stride; torch gives stride(0) = ldb
        return self.Bfull.as_strided((self.p.k, self.p.n), (self.p.ldb, 1)) if self.p.k and self.p.n else self.Bfull

    def _C_arg(self):
        return self.Cfull.as_strided((self.p.m, self.p.n), (self.ldc, 1)) if self.p.m and self.p.n else self.Cfull


def check_against_oracle(p, Cfull, ldc, *, exact=False, rows=None, label=""):
    """Element-by-element comparison with the fp64 oracle; also checks that padding columns kept the sentinel."""
    C = Cfull[:p.m, :p.n].astype(np.float64)
    C_ref, T = spmm_csr_oracle(p.m, p.n, p.rowptr, p.colidx, p.vals, p.B, p.ldb, rows=rows)
    if rows is not None:
        C = C[np.asarray(rows)]
    if exact:
        bad = C != C_ref
        assert not bad.any(), f"{label}: {int(bad.sum())} elements differ from the exact integer result; first at {np.argwhere(bad)[0]}"
        assert not np.signbit(C[C == 0]).any(), f"{label}: -0.0 where +0.0 is required"
    else:
        err = np.abs(C - C_ref)
        bound = RTOL_T * T + ATOL
        bad = ~(err <= bound)
        assert not bad.any(), (f"{label}: {int(bad.sum())} elements out of tolerance; worst err/bound = "
                               f"{np.nanmax(err / bound):.3g} at {np.argwhere(bad)[0]}")
    if ldc > p.n and p.m:
        assert np.all(Cfull[:p.m, p.n:] == SENTINEL), f"{label}: padding columns of C were written"
    return float(np.max(np.abs(C - C_ref) / (RTOL_T * T + ATOL))) if C.size else 0.0


def host_cores():
    """Worker threads for the chunked oracle: the CPU share of a one-GPU machine, never more than the affinity mask."""
    return max(1, min(16, len(os.sched_getaffinity(0))))


def check_every_row_chunked(p, outputs, *, exact=False, chunks_per_core=4):
    """Every element of one or more GPU results (dict label -> m x >=n float32 array) against the fp64 oracle.

    The oracle is the same serial loop as everywhere else; it is only called on contiguous blocks of rows, one block
    per call, several calls at a time on the host cores (ctypes releases the interpreter lock), and each block's
    C_ref and T are dropped after the comparison, so that the 2 x 8 bytes per element never exist for the whole matrix.
    Blocks hold about the same number of stored entries.  Returns the worst err/bound ratio per label."""
    from concurrent.futures import ThreadPoolExecutor

    cores = host_cores()
    rp = p.rowptr.astype(np.int64)
    nblocks = max(1, min(p.m, cores * chunks_per_core))
    cuts = np.searchsorted(rp, np.linspace(0, rp[-1], nblocks + 1)[1:-1], side="left")
    edges = np.unique(np.concatenate([[0], cuts, [p.m]])).astype(np.int64)
    for label, C in outputs.items():
        assert C.shape[0] >= p.m and C.shape[1] >= p.n, f"{label}: result has the wrong shape {C.shape}"

    def one(block):
        lo, hi = int(edges[block]), int(edges[block + 1])
        C_ref, T = spmm_csr_oracle(p.m, p.n, p.rowptr, p.colidx, p.vals, p.B, p.ldb, rows=np.arange(lo, hi, dtype=np.int64))
        res = {}
        for label, C in outputs.items():
            got = C[lo:hi, :p.n].astype(np.float64)
            if exact:
                bad = got != C_ref
                neg0 = bool(np.signbit(got[got == 0]).any())
                res[label] = (int(bad.sum()), (lo + int(np.argwhere(bad)[0][0])) if bad.any() else -1, 0.0, neg0)
            else:
                err = np.abs(got - C_ref)
                bound = RTOL_T * T + ATOL
                bad = ~(err <= bound)
                res[label] = (int(bad.sum()), (lo + int(np.argwhere(bad)[0][0])) if bad.any() else -1,
                              float(np.max(err / bound)) if err.size else 0.0, False)
        return res

    with ThreadPoolExecutor(max_workers=cores) as pool:
        parts = list(pool.map(one, range(len(edges) - 1)))
    worst = {}
    for label in outputs:
        nbad = sum(r[label][0] for r in parts)
        first = min([r[label][1] for r in parts if r[label][1] >= 0], default=-1)
        worst[label] = max(r[label][2] for r in parts)
        assert nbad == 0, (f"{label}: {nbad} elements " + ("differ from the exact integer result" if exact else
                           f"out of tolerance (worst err/bound {worst[label]:.3g})") + f"; first bad row {first}")
        assert not any(r[label][3] for r in parts), f"{label}: -0.0 where +0.0 is required"
    return worst


def read_plan_arrays(plan):
    """Copy the plan's lists out of the workspace (layout documented in the C header)."""
    info = plan.info()
    ws = plan.workspace.cpu().numpy()

    def view(off, count, width=1):
        return ws[off:off + count * width * 4].view(np.int32).reshape(count, width) if width > 1 else \
            ws[off:off + count * 4].view(np.int32)

    return info, {
        "win_row_start": view(info.off_win_row_start, info.n_windows + 1).copy(),
        "win_stage": view(info.off_win_stage, info.n_windows, 2).copy(),
        "wave_rows": view(info.off_wave_rows, info.n_wave_rows).copy(),
        "wave_span": view(info.off_wave_span, info.n_wave_rows, 2).copy(),
        "items": view(info.off_items, info.n_items, 4).copy(),
        "split": view(info.off_split, info.n_split_rows, 4).copy(),
    }
