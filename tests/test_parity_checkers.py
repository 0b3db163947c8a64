"""The comparison helpers of the GPU parity tests, exercised on the CPU: a result that equals the oracle's passes, and a
single wrong element anywhere -- one unit in the last place beyond the tolerance, a swapped pair of columns, a -0.0 in an
empty row -- fails.  (The mistakes are planted in host arrays; nothing here touches a GPU.)"""
import numpy as np
import pytest

from oracle import spmm_csr_oracle
from workloads import integer_valued, make_scaled_config

from gpu_util import ATOL, RTOL_T, check_every_row_chunked


@pytest.fixture(scope="module")
def problem():
    p = make_scaled_config(3, 0.02, seed=2)
    C_ref, T = spmm_csr_oracle(p.m, p.n, p.rowptr, p.colidx, p.vals, p.B, p.ldb)
    return p, C_ref, T


def test_oracle_result_rounded_to_fp32_passes(problem):
    p, C_ref, _ = problem
    worst = check_every_row_chunked(p, {"a": C_ref.astype(np.float32), "b": C_ref.astype(np.float32)})
    assert set(worst) == {"a", "b"} and all(0 <= w < 1 for w in worst.values())


@pytest.mark.parametrize("where", ["first", "last", "middle", "heaviest"])
def test_one_element_just_outside_the_tolerance_fails(problem, where):
    p, C_ref, T = problem
    C = C_ref.astype(np.float32)
    row = {"first": 0, "last": p.m - 1, "middle": p.m // 2, "heaviest": int(np.argmax(p.row_lengths))}[where]
    col = (7 * row) % p.n
    C[row, col] = np.float32(C_ref[row, col] + 2.5 * (RTOL_T * T[row, col] + ATOL))
    with pytest.raises(AssertionError, match="1 elements out of tolerance"):
        check_every_row_chunked(p, {"good": C_ref.astype(np.float32), "planted": C})


def test_two_swapped_columns_in_one_row_fail_although_the_row_sum_is_unchanged(problem):
    p, C_ref, _ = problem
    C = C_ref.astype(np.float32)
    row = int(np.argmax(p.row_lengths))
    C[row, [3, 4]] = C[row, [4, 3]]
    with pytest.raises(AssertionError, match="out of tolerance"):
        check_every_row_chunked(p, {"planted": C})


def test_exact_mode_wants_every_bit_and_positive_zero():
    p = integer_valued(make_scaled_config(1, 0.5, seed=1), seed=3)
    C_ref, _ = spmm_csr_oracle(p.m, p.n, p.rowptr, p.colidx, p.vals, p.B, p.ldb)
    good = C_ref.astype(np.float32)
    check_every_row_chunked(p, {"good": good}, exact=True)
    off = good.copy()
    off[p.m - 1, p.n - 1] += 1.0
    with pytest.raises(AssertionError, match="1 elements differ"):
        check_every_row_chunked(p, {"planted": off}, exact=True)
    zr, zc = np.argwhere(good == 0)[0]
    neg = good.copy()
    neg[zr, zc] = -0.0
    with pytest.raises(AssertionError, match="-0.0"):
        check_every_row_chunked(p, {"planted": neg}, exact=True)
