"""Pins of the fp64 SDDMM oracle (D = A (.) (B C) on the stored entries; paper Section 3.1) — no GPU needed."""
import os

import numpy as np
import pytest

from oracle import sddmm_csr_oracle
from workloads import csr_from_row_lengths, integer_valued, make_scaled_config

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def factors(m, k, d, seed, integer=False):
    rng = np.random.default_rng(seed)
    if integer:
        return (rng.integers(-8, 9, size=(m, d)).astype(np.float32), rng.integers(-8, 9, size=(k, d)).astype(np.float32))
    return rng.standard_normal((m, d)).astype(np.float32), rng.standard_normal((k, d)).astype(np.float32)


def test_handworked_fixture():
    d = {}
    for line in open(os.path.join(GOLDEN, "handworked_sddmm_3x3.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *rest = line.split()
        d[key] = rest
    m, k, dd = int(d["m"][0]), int(d["k"][0]), int(d["d"][0])
    D, T = sddmm_csr_oracle(m, dd, np.array(d["rowptr"], np.int32), np.array(d["colidx"], np.int32),
                            np.array(d["vals"], np.float32), np.array(d["B"], np.float32).reshape(m, dd),
                            np.array(d["Ct"], np.float32).reshape(k, dd))
    assert np.array_equal(D, np.array(d["D"], np.float64)) and np.array_equal(T, np.array(d["T"], np.float64))


@pytest.mark.parametrize("m,k,d,seed", [(1, 1, 1, 0), (9, 7, 5, 1), (40, 33, 64, 2), (17, 50, 130, 3)])
def test_dense_bruteforce_integer_exact(m, k, d, seed):
    rng = np.random.default_rng(seed)
    p = integer_valued(csr_from_row_lengths(rng.integers(0, min(k, 10) + 1, size=m), k, 4, seed=seed), seed=seed)
    B, Ct = factors(m, k, d, seed, integer=True)
    D, T = sddmm_csr_oracle(m, d, p.rowptr, p.colidx, p.vals, B, Ct)
    dense = B.astype(np.float64) @ Ct.astype(np.float64).T  # (B C) with C = Ct^T, m x k
    rows = np.repeat(np.arange(m), p.row_lengths)
    assert np.array_equal(D, p.vals.astype(np.float64) * dense[rows, p.colidx])
    # explicit loops, no BLAS, not transposed by accident: element (i, j) uses row i of B and row j of Ct
    for q in range(p.nnz):
        i, j = rows[q], p.colidx[q]
        s = 0.0
        for t in range(d):
            s += float(B[i, t]) * float(Ct[j, t])
        assert D[q] == float(p.vals[q]) * s
    assert np.array_equal(T, np.abs(p.vals.astype(np.float64)) * (np.abs(B).astype(np.float64) @ np.abs(Ct).astype(np.float64).T)[rows, p.colidx])


def test_dense_bruteforce_random_and_bounds():
    p = make_scaled_config(3, 0.01, seed=4)
    B, Ct = factors(p.m, p.k, 48, 5)
    D, T = sddmm_csr_oracle(p.m, 48, p.rowptr, p.colidx, p.vals, B, Ct)
    rows = np.repeat(np.arange(p.m), p.row_lengths)
    ref = p.vals.astype(np.float64) * np.einsum("pt,pt->p", B[rows].astype(np.float64), Ct[p.colidx].astype(np.float64))
    assert np.all(np.abs(D - ref) <= 1e-12 * T + 1e-300)
    assert np.all(T >= np.abs(D) * (1 - 1e-12))


def test_closed_forms():
    p = csr_from_row_lengths([3, 0, 5, 2], 9, 4, seed=6)
    d = 7
    ones_m, ones_k = np.ones((p.m, d), np.float32), np.ones((p.k, d), np.float32)
    D, _ = sddmm_csr_oracle(p.m, d, p.rowptr, p.colidx, p.vals, ones_m, ones_k)
    assert np.array_equal(D, p.vals.astype(np.float64) * d)  # all-ones factors: D = d * A
    # one-hot rows: B_i = e_(i mod d), Ct_j = e_(j mod d)  ->  D_ij = A_ij if i = j (mod d) else 0
    B = np.eye(d, dtype=np.float32)[np.arange(p.m) % d]
    Ct = np.eye(d, dtype=np.float32)[np.arange(p.k) % d]
    D, _ = sddmm_csr_oracle(p.m, d, p.rowptr, p.colidx, p.vals, B, Ct)
    rows = np.repeat(np.arange(p.m), p.row_lengths)
    assert np.array_equal(D, np.where(rows % d == p.colidx % d, p.vals.astype(np.float64), 0.0))


def test_linearity_in_each_factor_exact_on_integers():
    p = integer_valued(csr_from_row_lengths([4, 7, 0, 9], 12, 4, seed=7), seed=7)
    B1, Ct = factors(p.m, p.k, 16, 8, integer=True)
    B2, _ = factors(p.m, p.k, 16, 9, integer=True)
    D1, _ = sddmm_csr_oracle(p.m, 16, p.rowptr, p.colidx, p.vals, B1, Ct)
    D2, _ = sddmm_csr_oracle(p.m, 16, p.rowptr, p.colidx, p.vals, B2, Ct)
    D3, _ = sddmm_csr_oracle(p.m, 16, p.rowptr, p.colidx, p.vals, (B1 - 3 * B2).astype(np.float32), Ct)
    assert np.array_equal(D3, D1 - 3 * D2)


def test_padding_columns_are_never_read_and_empty_pattern():
    p = csr_from_row_lengths([3, 0, 5], 6, 4, seed=10)
    B, Ct = factors(p.m, p.k, 5, 11)
    D0, T0 = sddmm_csr_oracle(p.m, 5, p.rowptr, p.colidx, p.vals, B, Ct)
    Bp = np.full((p.m, 8), np.nan, np.float32)
    Bp[:, :5] = B
    Cp = np.full((p.k, 9), np.nan, np.float32)
    Cp[:, :5] = Ct
    D1, T1 = sddmm_csr_oracle(p.m, 5, p.rowptr, p.colidx, p.vals, Bp, Cp)
    assert np.array_equal(D0, D1) and np.array_equal(T0, T1)
    D, _ = sddmm_csr_oracle(4, 3, np.zeros(5, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32),
                            np.ones((4, 3), np.float32), np.ones((2, 3), np.float32))
    assert D.shape == (0,)
