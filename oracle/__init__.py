"""CPU oracles (test infrastructure only; never imported by the product package)."""
from .spmm import spmm_csr_oracle, spmm_bias_act_oracle, sddmm_csr_oracle, build_oracle, oracle_lib_path  # noqa: F401
from .plan import coo_rowptr_oracle, dcsr_rowptr_oracle, hot_columns_oracle, plan_oracle  # noqa: F401
