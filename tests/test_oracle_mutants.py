"""Shows that the pins have teeth: plausible slips planted in copies of the oracle source (on the CPU, in a
temporary directory) are each caught by at least one pin, while the unmodified source passes all of them."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "spmm_oracle.c")

# (name, text in the oracle source, replacement)
MUTANTS = [
    ("drops_last_entry_of_each_row", "p1 = rowptr[i + 1];", "p1 = rowptr[i + 1] - (rowptr[i + 1] > rowptr[i]);"),
    ("skips_first_entry_of_each_row", "for (int64_t p = p0; p < p1; ++p) {", "for (int64_t p = p0 + (p0 < p1); p < p1; ++p) {"),
    ("uses_row_pointer_of_previous_row", "int64_t p0 = rowptr[i], p1 = rowptr[i + 1];", "int64_t p0 = rowptr[i > 0 ? i - 1 : 0], p1 = rowptr[i + 1];"),
    ("adds_instead_of_multiplies", "c_row[c] += a * b;", "c_row[c] += a + b;"),
    ("overwrites_instead_of_accumulating", "c_row[c] += a * b;", "c_row[c] = a * b;"),
    ("wrong_sign", "c_row[c] += a * b;", "c_row[c] -= a * b;"),
    ("row_stride_of_B_is_n_not_ldb", "const float *b_row = B + (size_t)colidx[p] * (size_t)ldb;", "const float *b_row = B + (size_t)colidx[p] * (size_t)n;"),
    ("gathers_row_i_instead_of_column_index", "const float *b_row = B + (size_t)colidx[p] * (size_t)ldb;", "const float *b_row = B + (size_t)i * (size_t)ldb;"),
    ("product_rounded_to_single_precision", "c_row[c] += a * b;", "c_row[c] += (double)((float)a * (float)b);"),
    ("accumulator_rounded_to_single_precision", "c_row[c] += a * b;", "c_row[c] = (double)(float)(c_row[c] + a * b);"),
    ("tolerance_sum_without_absolute_values", "t_row[c] += fabs(a) * fabs(b);", "t_row[c] += a * b;"),
    ("row_subset_ignores_the_list", "int64_t i = rows ? rows[r] : r;", "int64_t i = r;"),
    ("accepts_out_of_range_row_ids", "if (i < 0 || i >= m) return -1;", "if (i < 0) return -1;"),
]


def compile_variant(tmp_path, name, old=None, new=None):
    text = open(SRC).read()
    if old is not None:
        assert text.count(old) == 1, f"mutation site for {name} not found exactly once"
        text = text.replace(old, new)
    c = tmp_path / f"{name}.c"
    so = tmp_path / f"{name}.so"
    c.write_text(text)
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"])
    lib = ctypes.CDLL(str(so))
    lib.spmm_csr_oracle.restype = ctypes.c_int
    lib.spmm_csr_oracle.argtypes = [ctypes.c_int64, ctypes.c_int64] + [ctypes.c_void_p] * 4 + \
        [ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
    return lib


def call(lib, m, n, rowptr, colidx, vals, B, rows=None):
    rowptr = np.ascontiguousarray(rowptr, np.int32)
    colidx = np.ascontiguousarray(colidx, np.int32)
    vals = np.ascontiguousarray(vals, np.float32)
    B = np.ascontiguousarray(B, np.float32)
    count = m if rows is None else len(rows)
    rows_a = None if rows is None else np.ascontiguousarray(rows, np.int64)
    C = np.full((count, n), 123.0)
    T = np.full((count, n), 123.0)
    rc = lib.spmm_csr_oracle(m, n, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data, B.ctypes.data, B.shape[1],
                             None if rows is None else rows_a.ctypes.data, count, C.ctypes.data, T.ctypes.data)
    return rc, C, T


def pins_pass(lib) -> bool:
    """A condensed copy of the pin suite; True when every check holds."""
    rng = np.random.default_rng(0)
    # hand-worked 3x3 (tests/golden/handworked_3x3.txt)
    rc, C, T = call(lib, 3, 2, [0, 2, 2, 3], [0, 2, 1], [1, 2, 3], np.array([[1, 2], [3, 4], [5, 6]]))
    if rc or not np.array_equal(C, [[11, 14], [0, 0], [9, 12]]) or not np.array_equal(T, [[11, 14], [0, 0], [9, 12]]):
        return False
    # dense brute force with negative values, m != k != n, leading dimension with NaN padding
    m, k, n, ldb = 9, 13, 5, 8
    A = np.where(rng.random((m, k)) < 0.3, rng.integers(-4, 5, size=(m, k)), 0).astype(np.float64)
    B = np.full((k, ldb), np.nan, np.float32)
    B[:, :n] = rng.integers(-8, 9, size=(k, n))
    rowptr = np.concatenate([[0], np.cumsum((A != 0).sum(axis=1))])
    colidx = np.concatenate([np.nonzero(A[i])[0] for i in range(m)])
    vals = np.concatenate([A[i][A[i] != 0] for i in range(m)])
    rc, C, T = call(lib, m, n, rowptr, colidx, vals, B)
    Bd = B[:, :n].astype(np.float64)
    if rc or not np.array_equal(C, A @ Bd) or not np.array_equal(T, np.abs(A) @ np.abs(Bd)):
        return False
    # row subset, and a row id out of range must be refused
    rc, Cs, _ = call(lib, m, n, rowptr, colidx, vals, B, rows=[m - 1, 2, 2])
    if rc or not np.array_equal(Cs, (A @ Bd)[[m - 1, 2, 2]]):
        return False
    # (rowptr gets two spare entries so that a variant without the range check reads valid memory)
    rc, _, _ = call(lib, m, n, np.concatenate([rowptr, rowptr[-1:], rowptr[-1:]]), colidx, vals, B, rows=[m])
    if rc == 0:
        return False
    # sequential fp64 accumulation in stored order: 2^60 + 1 - 2^60 = 0 in fp64 order, and 2^30 + 2^-30 is kept
    rc, C, _ = call(lib, 1, 1, [0, 3], [0, 1, 2], [2.0 ** 60, 1.0, -(2.0 ** 60)], np.ones((3, 1)))
    if rc or C[0, 0] != 0.0:
        return False
    rc, C, _ = call(lib, 1, 1, [0, 2], [0, 1], [2.0 ** 30, 2.0 ** -30], np.ones((2, 1)))
    if rc or C[0, 0] != 2.0 ** 30 + 2.0 ** -30:
        return False
    # a float*float product is exact in fp64: (1 + 2^-20)^2 = 1 + 2^-19 + 2^-40
    x = np.float32(1.0 + 2.0 ** -20)
    rc, C, _ = call(lib, 1, 1, [0, 1], [0], [x], np.array([[x]]))
    if rc or C[0, 0] != float(x) * float(x) or C[0, 0] == float(np.float32(x * x)):
        return False
    return True


def test_unmodified_oracle_passes_the_condensed_pins(tmp_path):
    assert pins_pass(compile_variant(tmp_path, "original"))


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    assert not pins_pass(compile_variant(tmp_path, name, old, new)), f"no pin notices the mutant '{name}'"


# ---- the SDDMM oracle (D_ij = A_ij * sum_t B_it C_tj on the stored entries; paper Section 3.1) ----
SRC_SDDMM = os.path.join(os.path.dirname(HERE), "oracle", "sddmm_oracle.c")

SDDMM_MUTANTS = [
    ("drops_last_entry_of_each_row", "int64_t p0 = rowptr[i], p1 = rowptr[i + 1];", "int64_t p0 = rowptr[i], p1 = rowptr[i + 1] - (rowptr[i + 1] > rowptr[i]);"),
    ("first_factor_row_is_the_column_index", "const float *b_row = B + (size_t)i * (size_t)ldb;", "const float *b_row = B + (size_t)(rowptr[i] < rowptr[i + 1] ? colidx[rowptr[i]] : 0) * (size_t)ldb;"),
    ("second_factor_row_is_the_row_index", "const float *c_row = Ct + (size_t)colidx[p] * (size_t)ldc;", "const float *c_row = Ct + (size_t)i * (size_t)ldc;"),
    ("second_factor_stride_is_ldb", "const float *c_row = Ct + (size_t)colidx[p] * (size_t)ldc;", "const float *c_row = Ct + (size_t)colidx[p] * (size_t)ldb;"),
    ("inner_sum_skips_the_last_term", "for (int64_t q = 0; q < d; ++q) {", "for (int64_t q = 0; q + 1 < d; ++q) {"),
    ("adds_instead_of_multiplies", "s += x * y;", "s += x + y;"),
    ("keeps_only_the_last_product", "s += x * y;", "s = x * y;"),
    ("forgets_the_value_of_A", "D[p] = (double)vals[p] * s;", "D[p] = s;"),
    ("adds_the_value_of_A", "D[p] = (double)vals[p] * s;", "D[p] = (double)vals[p] + s;"),
    ("wrong_sign", "D[p] = (double)vals[p] * s;", "D[p] = -(double)vals[p] * s;"),
    ("product_rounded_to_single_precision", "s += x * y;", "s += (double)((float)x * (float)y);"),
    ("sum_rounded_to_single_precision", "s += x * y;", "s = (double)(float)(s + x * y);"),
    ("tolerance_sum_without_absolute_values", "t += fabs(x) * fabs(y);", "t += x * y;"),
    ("tolerance_forgets_the_value_of_A", "if (T) T[p] = fabs((double)vals[p]) * t;", "if (T) T[p] = t;"),
]


def compile_sddmm_variant(tmp_path, name, old=None, new=None):
    text = open(SRC_SDDMM).read()
    if old is not None:
        assert text.count(old) == 1, f"mutation site for {name} not found exactly once"
        text = text.replace(old, new)
    c = tmp_path / f"sddmm_{name}.c"
    so = tmp_path / f"sddmm_{name}.so"
    c.write_text(text)
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"])
    lib = ctypes.CDLL(str(so))
    lib.sddmm_csr_oracle.restype = ctypes.c_int
    lib.sddmm_csr_oracle.argtypes = [ctypes.c_int64, ctypes.c_int64] + [ctypes.c_void_p] * 4 + \
        [ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
    return lib


def call_sddmm(lib, m, d, rowptr, colidx, vals, B, Ct):
    rowptr = np.ascontiguousarray(rowptr, np.int32)
    colidx = np.ascontiguousarray(colidx, np.int32)
    vals = np.ascontiguousarray(vals, np.float32)
    B = np.ascontiguousarray(B, np.float32)
    Ct = np.ascontiguousarray(Ct, np.float32)
    nnz = int(rowptr[-1])
    D = np.full(nnz, 123.0)
    T = np.full(nnz, 123.0)
    rc = lib.sddmm_csr_oracle(m, d, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data, B.ctypes.data, B.shape[1],
                              Ct.ctypes.data, Ct.shape[1], D.ctypes.data, T.ctypes.data)
    return rc, D, T


def sddmm_pins_pass(lib) -> bool:
    """A condensed copy of the SDDMM pin suite; True when every check holds."""
    rng = np.random.default_rng(1)
    # hand-worked values of tests/golden/handworked_sddmm_3x3.txt
    rc, D, T = call_sddmm(lib, 3, 2, [0, 2, 2, 3], [0, 2, 1], [2, -1, 0.5], [[1, 2], [3, 4], [5, 6]], [[1, 2], [0, 1], [-1, 3]])
    if rc or not np.array_equal(D, [10, -5, 3]) or not np.array_equal(T, [10, 7, 3]):
        return False
    # dense A (.) (B C) with m != k != d, negative values, padded leading dimensions filled with NaN
    m, k, d, ldb, ldc = 7, 11, 5, 8, 6
    A = np.where(rng.random((m, k)) < 0.35, rng.integers(-4, 5, size=(m, k)), 0).astype(np.float64)
    A[3] = 0
    B = np.full((m, ldb), np.nan, np.float32)
    B[:, :d] = rng.integers(-8, 9, size=(m, d))
    Ct = np.full((k, ldc), np.nan, np.float32)
    Ct[:, :d] = rng.integers(-8, 9, size=(k, d))
    rowptr = np.concatenate([[0], np.cumsum((A != 0).sum(axis=1))])
    colidx = np.concatenate([np.nonzero(A[i])[0] for i in range(m)])
    vals = np.concatenate([A[i][A[i] != 0] for i in range(m)])
    rows = np.repeat(np.arange(m), (A != 0).sum(axis=1))
    rc, D, T = call_sddmm(lib, m, d, rowptr, colidx, vals, B, Ct)
    Bd, Cd = B[:, :d].astype(np.float64), Ct[:, :d].astype(np.float64)
    if rc or not np.array_equal(D, vals * (Bd @ Cd.T)[rows, colidx]):
        return False
    if not np.array_equal(T, np.abs(vals) * (np.abs(Bd) @ np.abs(Cd).T)[rows, colidx]):
        return False
    # fp64 inner sum in index order: 2^60 + 1 - 2^60 = 0, and a float*float product is exact in fp64
    rc, D, _ = call_sddmm(lib, 1, 3, [0, 1], [0], [1.0], [[2.0 ** 60, 1.0, -(2.0 ** 60)]], [[1.0, 1.0, 1.0]])
    if rc or D[0] != 0.0:
        return False
    rc, D, _ = call_sddmm(lib, 1, 2, [0, 1], [0], [1.0], [[2.0 ** 30, 2.0 ** -30]], [[1.0, 1.0]])
    if rc or D[0] != 2.0 ** 30 + 2.0 ** -30:
        return False
    x = np.float32(1.0 + 2.0 ** -20)
    rc, D, _ = call_sddmm(lib, 1, 1, [0, 1], [0], [1.0], [[x]], [[x]])
    if rc or D[0] != float(x) * float(x) or D[0] == float(np.float32(x * x)):
        return False
    return True


def test_unmodified_sddmm_oracle_passes_the_condensed_pins(tmp_path):
    assert sddmm_pins_pass(compile_sddmm_variant(tmp_path, "original"))


@pytest.mark.parametrize("name,old,new", SDDMM_MUTANTS, ids=[m[0] for m in SDDMM_MUTANTS])
def test_planted_mistake_in_the_sddmm_oracle_is_caught(tmp_path, name, old, new):
    assert not sddmm_pins_pass(compile_sddmm_variant(tmp_path, name, old, new)), f"no pin notices the mutant '{name}'"
