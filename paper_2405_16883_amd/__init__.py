"""MI355X-native CSR SpMM (C = A.B, A sparse CSR, B and C dense fp32) behind a C ABI.

The product is libscorch_spmm.so (hand-written HIP for gfx950, see csrc/ and include/scorch_spmm.h);
this package is its ctypes binding.
"""
from .binding import (  # noqa: F401
    EXPORTS, LIB_PATH, PlanInfo, ScorchError, SpmmPlan, load_library, scorch_spmm_csr, scorch_spmm_csr_planned,
    scorch_spmm_plan, scorch_spmm_plan_workspace_bytes, scorch_sddmm_csr, scorch_sddmm_csr_planned, scorch_spmm_csr_planned_epilogue, scorch_coo_to_csr_rowptr, scorch_dcsr_to_csr_rowptr, ACT_IDENTITY, ACT_RELU,
    scorch_spmm_csr_static, STATIC_SCRATCH_BYTES,
)
