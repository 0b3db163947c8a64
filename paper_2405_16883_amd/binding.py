"""Thin ctypes binding of the C ABI in include/scorch_spmm.h.

Argument marshalling only: every step of the SpMM path runs inside libscorch_spmm.so.  torch is
used for device memory and streams.  There is no fallback: if the library is missing or a call
fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libscorch_spmm.so")

SCORCH_OK = 0
SCORCH_ERR_INVALID_ARG = -1
SCORCH_ERR_UNSUPPORTED = -2
SCORCH_ERR_WORKSPACE_TOO_SMALL = -3
SCORCH_ERR_HIP = -4

EXPORTS = (
    "scorch_spmm_csr", "scorch_spmm_plan_workspace_bytes", "scorch_spmm_plan", "scorch_spmm_csr_planned",
    "scorch_spmm_plan_destroy", "scorch_spmm_plan_info", "scorch_status_string", "scorch_last_error",
    "scorch_sddmm_csr", "scorch_sddmm_csr_planned", "scorch_spmm_csr_planned_epilogue", "scorch_coo_to_csr_rowptr",
    "scorch_dcsr_to_csr_rowptr", "scorch_spmm_csr_static",
)


class ScorchError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"scorch status {status}: {message}")
        self.status = status


class PlanInfo(ctypes.Structure):
    _fields_ = [
        ("m", ctypes.c_int32), ("k", ctypes.c_int32), ("n", ctypes.c_int32), ("nnz", ctypes.c_int64),
        ("BN", ctypes.c_int32), ("ALPHA", ctypes.c_int32), ("LW", ctypes.c_int32), ("CH", ctypes.c_int32),
        ("BCH", ctypes.c_int32),
        ("n_windows", ctypes.c_int32), ("n_short_rows", ctypes.c_int32), ("n_wave_rows", ctypes.c_int32),
        ("n_items", ctypes.c_int32), ("n_split_rows", ctypes.c_int32), ("n_partial_slots", ctypes.c_int32),
        ("partial_stride", ctypes.c_int32), ("mode", ctypes.c_int32),
        ("off_win_row_start", ctypes.c_uint64), ("off_wave_rows", ctypes.c_uint64), ("off_items", ctypes.c_uint64),
        ("off_split", ctypes.c_uint64), ("off_partials", ctypes.c_uint64), ("workspace_bytes_used", ctypes.c_uint64),
        ("n_hot_columns", ctypes.c_int32), ("hot_share", ctypes.c_float), ("off_wave_span", ctypes.c_uint64), ("off_win_stage", ctypes.c_uint64),
    ]


_lib = None


def load_library() -> ctypes.CDLL:
    """dlopen the in-tree library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2405_16883_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    i32, i64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
    lib.scorch_spmm_csr.restype = i32
    lib.scorch_spmm_csr.argtypes = [i32, i32, i32, vp, vp, vp, vp, i32, vp, i32, vp]
    lib.scorch_spmm_csr_static.restype = i32
    lib.scorch_spmm_csr_static.argtypes = [i32, i32, i32, vp, vp, vp, vp, i32, vp, i32, vp]
    lib.scorch_spmm_plan_workspace_bytes.restype = i32
    lib.scorch_spmm_plan_workspace_bytes.argtypes = [i32, i32, i32, i64, ctypes.POINTER(ctypes.c_size_t)]
    lib.scorch_spmm_plan.restype = i32
    lib.scorch_spmm_plan.argtypes = [i32, i32, i32, vp, vp, vp, ctypes.c_size_t, vp, ctypes.POINTER(vp)]
    lib.scorch_spmm_csr_planned.restype = i32
    lib.scorch_spmm_csr_planned.argtypes = [vp, vp, vp, vp, vp, i32, vp, i32, vp]
    lib.scorch_spmm_plan_destroy.restype = i32
    lib.scorch_spmm_plan_destroy.argtypes = [vp]
    lib.scorch_spmm_plan_info.restype = i32
    lib.scorch_spmm_plan_info.argtypes = [vp, ctypes.POINTER(PlanInfo)]
    lib.scorch_spmm_csr_planned_epilogue.restype = i32
    lib.scorch_spmm_csr_planned_epilogue.argtypes = [vp, vp, vp, vp, vp, i32, vp, i32, vp, i32, vp]
    lib.scorch_coo_to_csr_rowptr.restype = i32
    lib.scorch_coo_to_csr_rowptr.argtypes = [i32, i64, vp, vp, vp, vp]
    lib.scorch_dcsr_to_csr_rowptr.restype = i32
    lib.scorch_dcsr_to_csr_rowptr.argtypes = [i32, i32, vp, vp, vp, vp, vp]
    lib.scorch_sddmm_csr.restype = i32
    lib.scorch_sddmm_csr.argtypes = [i32, i32, i32, vp, vp, vp, vp, i32, vp, i32, vp, vp]
    lib.scorch_sddmm_csr_planned.restype = i32
    lib.scorch_sddmm_csr_planned.argtypes = [vp, i32, vp, vp, vp, vp, i32, vp, i32, vp, vp]
    lib.scorch_status_string.restype = ctypes.c_char_p
    lib.scorch_status_string.argtypes = [i32]
    lib.scorch_last_error.restype = ctypes.c_char_p
    lib.scorch_last_error.argtypes = []
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != SCORCH_OK:
        lib = load_library()
        raise ScorchError(status, f"{lib.scorch_status_string(status).decode()}: {lib.scorch_last_error().decode()}")


def _dev_ptr(t: Optional[torch.Tensor], dtype: torch.dtype, name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr() if t.numel() else None


def _ld(t: torch.Tensor, name: str) -> int:
    if t.dim() != 2 or (t.numel() and t.stride(1) != 1):
        raise ValueError(f"{name} must be 2-D with unit column stride")
    return int(t.stride(0)) if t.shape[0] > 1 else max(int(t.stride(0)), int(t.shape[1]))


def _stream_handle(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def scorch_spmm_csr(m: int, k: int, n: int, rowptr: torch.Tensor, colidx: torch.Tensor, vals: torch.Tensor,
                    B: torch.Tensor, C: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    """C[:m, :n] = A @ B[:k, :n] through the plan-free entry point.  B and C may be row-strided views."""
    lib = load_library()
    _check(lib.scorch_spmm_csr(m, k, n, _dev_ptr(rowptr, torch.int32, "rowptr"), _dev_ptr(colidx, torch.int32, "colidx"),
                               _dev_ptr(vals, torch.float32, "vals"), _dev_ptr(B, torch.float32, "B"), _ld(B, "B"),
                               _dev_ptr(C, torch.float32, "C"), _ld(C, "C"), _stream_handle(stream)))


STATIC_SCRATCH_BYTES = 16 << 20


def scorch_spmm_csr_static(m: int, k: int, n: int, rowptr: torch.Tensor, colidx: torch.Tensor, vals: torch.Tensor,
                           B: torch.Tensor, C: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    """C[:m, :n] = A @ B[:k, :n] through the entry point that allocates nothing on the device (the plan lives in the
    library's static scratch array; problems whose plan needs more than STATIC_SCRATCH_BYTES are refused)."""
    lib = load_library()
    _check(lib.scorch_spmm_csr_static(m, k, n, _dev_ptr(rowptr, torch.int32, "rowptr"), _dev_ptr(colidx, torch.int32, "colidx"),
                                      _dev_ptr(vals, torch.float32, "vals"), _dev_ptr(B, torch.float32, "B"), _ld(B, "B"),
                                      _dev_ptr(C, torch.float32, "C"), _ld(C, "C"), _stream_handle(stream)))


def scorch_spmm_plan_workspace_bytes(m: int, k: int, n: int, nnz: int) -> int:
    lib = load_library()
    out = ctypes.c_size_t(0)
    _check(lib.scorch_spmm_plan_workspace_bytes(m, k, n, nnz, ctypes.byref(out)))
    return int(out.value)


class SpmmPlan:
    """Owns the C plan handle and the torch tensor that backs its device workspace."""

    def __init__(self, handle: int, workspace: torch.Tensor):
        self._handle = handle
        self.workspace = workspace

    @property
    def handle(self) -> int:
        if not self._handle:
            raise ValueError("plan already destroyed")
        return self._handle

    def info(self) -> PlanInfo:
        out = PlanInfo()
        _check(load_library().scorch_spmm_plan_info(self.handle, ctypes.byref(out)))
        return out

    def destroy(self) -> None:
        if self._handle:
            load_library().scorch_spmm_plan_destroy(self._handle)
            self._handle = 0

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def scorch_spmm_plan(m: int, k: int, n: int, rowptr: torch.Tensor, nnz: int,
                     colidx: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None,
                     stream: Optional[torch.cuda.Stream] = None) -> SpmmPlan:
    """Analyse the pattern behind ``rowptr`` (and, if given, ``colidx``).  ``workspace`` (uint8, GPU) is allocated
    with torch if not given."""
    lib = load_library()
    if workspace is None:
        workspace = torch.empty(scorch_spmm_plan_workspace_bytes(m, k, n, nnz), dtype=torch.uint8, device=rowptr.device)
    handle = ctypes.c_void_p(0)
    _check(lib.scorch_spmm_plan(m, k, n, _dev_ptr(rowptr, torch.int32, "rowptr"), _dev_ptr(colidx, torch.int32, "colidx"),
                                _dev_ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
                                _stream_handle(stream), ctypes.byref(handle)))
    return SpmmPlan(handle.value, workspace)


def scorch_spmm_csr_planned(plan: SpmmPlan, rowptr: torch.Tensor, colidx: torch.Tensor, vals: torch.Tensor,
                            B: torch.Tensor, C: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    lib = load_library()
    _check(lib.scorch_spmm_csr_planned(plan.handle, _dev_ptr(rowptr, torch.int32, "rowptr"),
                                       _dev_ptr(colidx, torch.int32, "colidx"), _dev_ptr(vals, torch.float32, "vals"),
                                       _dev_ptr(B, torch.float32, "B"), _ld(B, "B"),
                                       _dev_ptr(C, torch.float32, "C"), _ld(C, "C"), _stream_handle(stream)))


def scorch_sddmm_csr(m: int, k: int, d: int, rowptr: torch.Tensor, colidx: torch.Tensor, vals: torch.Tensor,
                     B: torch.Tensor, Ct: torch.Tensor, out_vals: torch.Tensor,
                     stream: Optional[torch.cuda.Stream] = None) -> None:
    """out_vals[p] = vals[p] * <B[i, :d], Ct[colidx[p], :d]> through the plan-free entry point."""
    lib = load_library()
    _check(lib.scorch_sddmm_csr(m, k, d, _dev_ptr(rowptr, torch.int32, "rowptr"), _dev_ptr(colidx, torch.int32, "colidx"),
                                _dev_ptr(vals, torch.float32, "vals"), _dev_ptr(B, torch.float32, "B"), _ld(B, "B"),
                                _dev_ptr(Ct, torch.float32, "Ct"), _ld(Ct, "Ct"),
                                _dev_ptr(out_vals, torch.float32, "out_vals"), _stream_handle(stream)))


def scorch_sddmm_csr_planned(plan: SpmmPlan, d: int, rowptr: torch.Tensor, colidx: torch.Tensor, vals: torch.Tensor,
                             B: torch.Tensor, Ct: torch.Tensor, out_vals: torch.Tensor,
                             stream: Optional[torch.cuda.Stream] = None) -> None:
    lib = load_library()
    _check(lib.scorch_sddmm_csr_planned(plan.handle, d, _dev_ptr(rowptr, torch.int32, "rowptr"),
                                        _dev_ptr(colidx, torch.int32, "colidx"), _dev_ptr(vals, torch.float32, "vals"),
                                        _dev_ptr(B, torch.float32, "B"), _ld(B, "B"), _dev_ptr(Ct, torch.float32, "Ct"),
                                        _ld(Ct, "Ct"), _dev_ptr(out_vals, torch.float32, "out_vals"),
                                        _stream_handle(stream)))


ACT_IDENTITY = 0
ACT_RELU = 1


def scorch_spmm_csr_planned_epilogue(plan: SpmmPlan, rowptr: torch.Tensor, colidx: torch.Tensor, vals: torch.Tensor,
                                     B: torch.Tensor, bias: Optional[torch.Tensor], activation: int, C: torch.Tensor,
                                     stream: Optional[torch.cuda.Stream] = None) -> None:
    """C = act(A @ B + bias) in one pass (bias may be None; activation ACT_IDENTITY or ACT_RELU)."""
    lib = load_library()
    _check(lib.scorch_spmm_csr_planned_epilogue(plan.handle, _dev_ptr(rowptr, torch.int32, "rowptr"),
                                                _dev_ptr(colidx, torch.int32, "colidx"),
                                                _dev_ptr(vals, torch.float32, "vals"), _dev_ptr(B, torch.float32, "B"),
                                                _ld(B, "B"), _dev_ptr(bias, torch.float32, "bias"), activation,
                                                _dev_ptr(C, torch.float32, "C"), _ld(C, "C"), _stream_handle(stream)))


def scorch_coo_to_csr_rowptr(m: int, row_idx: torch.Tensor, rowptr_out: torch.Tensor,
                             bad_flag: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> None:
    """rowptr_out[0..m] for a coordinate list whose int32 row coordinates ``row_idx`` are sorted by row."""
    lib = load_library()
    if rowptr_out.numel() != m + 1:
        raise ValueError("rowptr_out must have m + 1 entries")
    _check(lib.scorch_coo_to_csr_rowptr(m, row_idx.numel(), _dev_ptr(row_idx, torch.int32, "row_idx"),
                                        _dev_ptr(rowptr_out, torch.int32, "rowptr_out"),
                                        _dev_ptr(bad_flag, torch.int32, "bad_flag"), _stream_handle(stream)))


def scorch_dcsr_to_csr_rowptr(m: int, row_ids: torch.Tensor, row_pos: torch.Tensor, rowptr_out: torch.Tensor,
                              bad_flag: Optional[torch.Tensor] = None,
                              stream: Optional[torch.cuda.Stream] = None) -> None:
    """CSR row pointers of a doubly compressed matrix given the ids of its stored rows and their entry ranges."""
    lib = load_library()
    if rowptr_out.numel() != m + 1 or row_pos.numel() != row_ids.numel() + 1:
        raise ValueError("rowptr_out needs m + 1 entries and row_pos one more entry than row_ids")
    _check(lib.scorch_dcsr_to_csr_rowptr(m, row_ids.numel(), _dev_ptr(row_ids, torch.int32, "row_ids"),
                                         row_pos.data_ptr(), _dev_ptr(rowptr_out, torch.int32, "rowptr_out"),
                                         _dev_ptr(bad_flag, torch.int32, "bad_flag"), _stream_handle(stream)))
