"""ctypes front end of the plain-C fp64 SpMM oracle (oracle/spmm_oracle.c).

TEST INFRASTRUCTURE ONLY.  Importers allowed: tests/, the smoke check and the cpu_baseline
leg of the benchmark.  It shares no code with the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spmm_oracle.c")
_SRC2 = os.path.join(_HERE, "sddmm_oracle.c")
_LIB = os.path.join(_HERE, "libspmm_oracle.so")
_lib = None


def oracle_lib_path() -> str:
    return _LIB


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, strict IEEE: no -ffast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_SRC2)):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fPIC", "-shared",
                               "-o", tmp, _SRC, _SRC2, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build_oracle()
        lib = ctypes.CDLL(_LIB)
        lib.spmm_csr_oracle.restype = ctypes.c_int
        lib.spmm_csr_oracle.argtypes = [ctypes.c_int64, ctypes.c_int64] + [ctypes.c_void_p] * 4 + \
            [ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
        lib.sddmm_csr_oracle.restype = ctypes.c_int
        lib.sddmm_csr_oracle.argtypes = [ctypes.c_int64, ctypes.c_int64] + [ctypes.c_void_p] * 4 + \
            [ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
        _lib = lib
    return _lib


def sddmm_csr_oracle(m: int, d: int, rowptr: np.ndarray, colidx: np.ndarray, vals: np.ndarray,
                     B: np.ndarray, Ct: np.ndarray, want_T: bool = True):
    """D_p = vals[p] * <B[i,:d], Ct[colidx[p],:d]> in fp64 for every stored entry p of row i, and its magnitude sum.

    ``B`` is m x ldb and ``Ct`` (the second factor, transposed) k x ldc, both float32 row-major.
    """
    lib = _load()
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    B = np.ascontiguousarray(B, dtype=np.float32)
    Ct = np.ascontiguousarray(Ct, dtype=np.float32)
    nnz = int(rowptr[-1])
    assert rowptr.shape[0] == m + 1 and B.shape[0] >= m and B.shape[1] >= d and Ct.shape[1] >= d
    if nnz:
        assert int(colidx[:nnz].min()) >= 0 and int(colidx[:nnz].max()) < Ct.shape[0]
    D = np.empty(nnz, dtype=np.float64)
    T = np.empty(nnz, dtype=np.float64) if want_T else None
    rc = lib.sddmm_csr_oracle(m, d, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data,
                              B.ctypes.data, B.shape[1], Ct.ctypes.data, Ct.shape[1], D.ctypes.data,
                              T.ctypes.data if want_T else None)
    if rc != 0:
        raise ValueError("sddmm_csr_oracle: malformed CSR")
    return D, T


def spmm_csr_oracle(m: int, n: int, rowptr: np.ndarray, colidx: np.ndarray, vals: np.ndarray,
                    B: np.ndarray, ldb: Optional[int] = None, rows: Optional[np.ndarray] = None,
                    want_T: bool = True) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """C_ref (fp64) and, if asked, T = |A|.|B| (fp64) for all rows or for the listed ``rows``.

    ``B`` is a float32 array holding k rows of stride ``ldb`` (default: its second dimension).
    """
    lib = _load()
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    B = np.ascontiguousarray(B, dtype=np.float32)
    if ldb is None:
        ldb = B.shape[1] if B.ndim == 2 else n
    assert rowptr.shape[0] == m + 1
    nnz = int(rowptr[-1])
    assert colidx.shape[0] >= nnz and vals.shape[0] >= nnz and ldb >= n
    if nnz:
        kmax = int(colidx[:nnz].max())
        assert int(colidx[:nnz].min()) >= 0 and (kmax + 1) * ldb <= B.size + (ldb - n)
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        count = rows.shape[0]
        rows_p = rows.ctypes.data
    else:
        count = m
        rows_p = None
    C = np.empty((count, n), dtype=np.float64)
    T = np.empty((count, n), dtype=np.float64) if want_T else None
    rc = lib.spmm_csr_oracle(m, n, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data,
                             B.ctypes.data, ldb, rows_p, count, C.ctypes.data,
                             T.ctypes.data if want_T else None)
    if rc != 0:
        raise ValueError("spmm_csr_oracle: malformed CSR or row list")
    return C, T


def spmm_bias_act_oracle(m: int, n: int, rowptr, colidx, vals, B, bias, relu: bool, ldb: Optional[int] = None,
                         rows: Optional[np.ndarray] = None):
    """GCN-style layer output (paper, Section 5.1: H' = sigma(A^ H W)), evaluated as sigma(A^ (H W) + b):
    C_ik = act(sum_j A_ij B_jk + bias_k) in fp64, with B standing for H W.  The SpMM part is the plain oracle
    above; bias and max(., 0) are applied to its fp64 result.  Also returns the magnitude sum T + |bias|."""
    C, T = spmm_csr_oracle(m, n, rowptr, colidx, vals, B, ldb, rows=rows)
    if bias is not None:
        b = np.asarray(bias, dtype=np.float32).astype(np.float64)
        C = C + b[None, :]
        T = T + np.abs(b)[None, :]
    if relu:
        C = np.maximum(C, 0.0)
    return C, T
