"""Seeded synthetic operands for CSR SpMM (C = A.B, A sparse m x k, B dense k x n).

This package only *draws inputs*.  It contains none of the SpMM arithmetic, no
planner logic and no kernels, and it imports neither the CPU oracle nor the HIP
library, so both sides of a parity test can be fed from it.
"""
from .generators import (  # noqa: F401
    SpmmProblem,
    CONFIG_NAMES,
    make_config,
    make_scaled_config,
    tiny_powerlaw,
    uniform_rows,
    chung_lu_graph,
    pruned_weight,
    csr_from_row_lengths,
    integer_valued,
    with_padding,
    count_unique_columns,
    min_traffic_bytes,
)
