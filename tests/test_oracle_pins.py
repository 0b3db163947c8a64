"""Pins of the fp64 CPU oracle to things other than itself (runs without a GPU).

The oracle states C_ik = sum_j A_ij B_jk over the stored entries of a CSR row (paper, Section 4.2
SpMM example; CSR per Appendix C).  Each test below would fail for a plausible slip in it: a
dropped or doubled term, a sign, a transposed or mis-strided operand, an off-by-one row pointer.
"""
import os

import numpy as np
import pytest

from oracle import spmm_bias_act_oracle, spmm_csr_oracle
from workloads import (csr_from_row_lengths, integer_valued, make_scaled_config, tiny_powerlaw,
                       uniform_rows, with_padding)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def densify(p):
    """Dense fp64 copy of A; repeated (row, col) entries add up, as the definition sums stored entries."""
    A = np.zeros((p.m, p.k), dtype=np.float64)
    rows = np.repeat(np.arange(p.m), p.row_lengths)
    np.add.at(A, (rows, p.colidx.astype(np.int64)), p.vals.astype(np.float64))
    return A


def oracle(p, **kw):
    return spmm_csr_oracle(p.m, p.n, p.rowptr, p.colidx, p.vals, p.B, p.ldb, **kw)


def read_fixture(name):
    d = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *rest = line.split()
            d[key] = rest
    m, k, n = int(d["m"][0]), int(d["k"][0]), int(d["n"][0])
    return dict(m=m, k=k, n=n,
                rowptr=np.array(d["rowptr"], dtype=np.int32), colidx=np.array(d["colidx"], dtype=np.int32),
                vals=np.array(d["vals"], dtype=np.float32), B=np.array(d["B"], dtype=np.float32).reshape(k, n),
                C=np.array(d["C"], dtype=np.float64).reshape(m, n), T=np.array(d["T"], dtype=np.float64).reshape(m, n))


@pytest.mark.parametrize("name", ["handworked_3x3.txt", "handworked_signs_4x5.txt"])
def test_handworked_fixture(name):
    g = read_fixture(name)
    C, T = spmm_csr_oracle(g["m"], g["n"], g["rowptr"], g["colidx"], g["vals"], g["B"])
    assert np.array_equal(C, g["C"])
    assert np.array_equal(T, g["T"])


@pytest.mark.parametrize("m,k,n,seed", [(1, 1, 1, 0), (7, 5, 3, 1), (33, 64, 17, 2), (64, 40, 65, 3)])
def test_dense_bruteforce_integer_exact(m, k, n, seed):
    rng = np.random.default_rng(seed)
    lens = rng.integers(0, min(k, 12) + 1, size=m)
    p = integer_valued(csr_from_row_lengths(lens, k, n, seed=seed), seed=seed)
    A = densify(p)
    Bd = p.B[:, :n].astype(np.float64)
    # explicit triple loop, independent of both the oracle and of BLAS
    ref = np.zeros((m, n))
    for i in range(m):
        for j in range(k):
            if A[i, j] != 0.0:
                for c in range(n):
                    ref[i, c] += A[i, j] * Bd[j, c]
    C, T = oracle(p)
    assert np.array_equal(C, ref)
    assert np.array_equal(C, A @ Bd)  # integers: any summation order is exact
    assert np.array_equal(T, np.abs(A) @ np.abs(Bd))


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_dense_bruteforce_random(seed):
    rng = np.random.default_rng(100 + seed)
    m, k, n = 48, 56, 29
    p = csr_from_row_lengths(rng.integers(0, 30, size=m), k, n, seed=seed)
    C, T = oracle(p)
    ref = densify(p) @ p.B[:, :n].astype(np.float64)
    assert np.all(np.abs(C - ref) <= 1e-12 * T + 1e-300)
    assert np.all(T >= np.abs(C) * (1 - 1e-12))


def test_identity_and_permutation_bit_exact():
    k, n = 37, 19
    B = np.random.default_rng(5).standard_normal((k, n)).astype(np.float32)
    rowptr = np.arange(k + 1, dtype=np.int32)
    ones = np.ones(k, dtype=np.float32)
    C, _ = spmm_csr_oracle(k, n, rowptr, np.arange(k, dtype=np.int32), ones, B)
    assert np.array_equal(C, B.astype(np.float64))
    pi = np.random.default_rng(6).permutation(k).astype(np.int32)
    C, _ = spmm_csr_oracle(k, n, rowptr, pi, ones, B)
    assert np.array_equal(C, B[pi].astype(np.float64))  # row i of C is row pi(i) of B, not the inverse
    scale = (2.0 ** np.random.default_rng(7).integers(-6, 7, size=k)).astype(np.float32)
    scale *= np.where(np.arange(k) % 2 == 0, 1.0, -1.0).astype(np.float32)
    C, T = spmm_csr_oracle(k, n, rowptr, pi, scale, B)
    assert np.array_equal(C, scale[:, None].astype(np.float64) * B[pi].astype(np.float64))
    assert np.array_equal(T, np.abs(C))


def test_rectangular_shapes_not_transposed():
    # m != k != n and a B whose rows are recognisable: entry (j, c) = 1000*j + c
    m, k, n = 5, 9, 4
    B = (1000.0 * np.arange(k)[:, None] + np.arange(n)[None, :]).astype(np.float32)
    rowptr = np.array([0, 1, 1, 3, 4, 6], dtype=np.int32)
    colidx = np.array([8, 0, 7, 3, 2, 5], dtype=np.int32)
    vals = np.array([1, 1, 2, -1, 3, 1], dtype=np.float32)
    C, _ = spmm_csr_oracle(m, n, rowptr, colidx, vals, B)
    expect = np.array([B[8], 0 * B[0], B[0] + 2 * B[7], -B[3], 3 * B[2] + B[5]], dtype=np.float64)
    assert np.array_equal(C, expect)


def test_row_sum_invariant():
    p = make_scaled_config(3, 0.01, seed=3)
    C, T = oracle(p)
    b1 = p.B[:, :p.n].astype(np.float64).sum(axis=1)
    rows = np.repeat(np.arange(p.m), p.row_lengths)
    lhs = C.sum(axis=1)
    rhs = np.zeros(p.m)
    np.add.at(rhs, rows, p.vals.astype(np.float64) * b1[p.colidx])
    assert np.all(np.abs(lhs - rhs) <= 1e-12 * T.sum(axis=1) + 1e-300)


def test_against_int64_arithmetic():
    p = integer_valued(make_scaled_config(4, 0.0008, seed=1), seed=1)
    C, T = oracle(p)
    Bi = p.B[:, :p.n].astype(np.int64)
    vi = p.vals.astype(np.int64)
    ref = np.zeros((p.m, p.n), dtype=np.int64)
    for i in range(p.m):
        for q in range(p.rowptr[i], p.rowptr[i + 1]):
            ref[i] += vi[q] * Bi[p.colidx[q]]
    assert np.array_equal(C, ref.astype(np.float64))
    assert np.all(C == np.round(C))


def test_linearity_exact_on_integers():
    p1 = integer_valued(tiny_powerlaw(m=200, n=16, seed=4), seed=10)
    p2 = integer_valued(tiny_powerlaw(m=200, n=16, seed=4), seed=11)
    B3 = (p1.B + 2.0 * p2.B).astype(np.float32)
    C1, _ = oracle(p1)
    C2, _ = spmm_csr_oracle(p1.m, p1.n, p1.rowptr, p1.colidx, p1.vals, p2.B)
    C3, _ = spmm_csr_oracle(p1.m, p1.n, p1.rowptr, p1.colidx, p1.vals, B3)
    assert np.array_equal(C3, C1 + 2.0 * C2)


def test_column_independence_bit_exact():
    p = uniform_rows(m=64, k=300, density=0.05, n=9, seed=8)
    C, T = oracle(p)
    for c in (0, 4, 8):
        col = np.ascontiguousarray(p.B[:, c:c + 1])
        Cc, Tc = spmm_csr_oracle(p.m, 1, p.rowptr, p.colidx, p.vals, col, 1)
        assert np.array_equal(Cc[:, 0], C[:, c]) and np.array_equal(Tc[:, 0], T[:, c])


def test_all_ones_gives_column_sums():
    m, k, n = 6, 23, 7
    B = np.random.default_rng(9).integers(-8, 9, size=(k, n)).astype(np.float32)
    rowptr = (np.arange(m + 1) * k).astype(np.int32)
    colidx = np.tile(np.arange(k, dtype=np.int32), m)
    C, _ = spmm_csr_oracle(m, n, rowptr, colidx, np.ones(m * k, np.float32), B)
    assert np.array_equal(C, np.tile(B.astype(np.float64).sum(axis=0), (m, 1)))


def test_leading_dimension_padding_is_never_read():
    p = csr_from_row_lengths([3, 0, 5, 1], 11, 6, seed=12)
    C0, T0 = oracle(p)
    pp = with_padding(p, ldb=10)  # padding columns hold NaN
    C1, T1 = oracle(pp)
    assert np.array_equal(C0, C1) and np.array_equal(T0, T1)
    assert np.all(np.isfinite(C1))


def test_duplicates_and_unsorted_columns_sum_stored_entries():
    p = csr_from_row_lengths([40, 7, 0, 25], 12, 5, seed=13, sorted_cols=False, duplicates=True)
    assert len(np.unique(p.colidx[:40])) < 40
    C, T = oracle(p)
    ref = densify(p) @ p.B[:, :p.n].astype(np.float64)
    assert np.all(np.abs(C - ref) <= 1e-12 * T)


def test_empty_rows_and_edge_shapes():
    # all rows empty
    C, T = spmm_csr_oracle(4, 3, np.zeros(5, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32),
                           np.ones((2, 3), np.float32))
    assert C.shape == (4, 3) and not C.any() and not T.any()
    assert not np.signbit(C).any()  # +0.0
    # m = 0
    C, _ = spmm_csr_oracle(0, 3, np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32),
                           np.ones((2, 3), np.float32))
    assert C.shape == (0, 3)
    # last row empty, first row heavy, k = 1
    p = csr_from_row_lengths([500, 1, 0], 1, 4, seed=14, duplicates=True)
    C, _ = oracle(p)
    assert np.allclose(C[0], p.vals[:500].astype(np.float64).sum() * p.B[0, :4].astype(np.float64), rtol=1e-12, atol=1e-12)
    assert not C[2].any()


def test_row_subset_matches_full():
    p = make_scaled_config(1, 0.1, seed=2)
    C, T = oracle(p)
    rows = np.array([p.m - 1, 0, 17, 17, 3], dtype=np.int64)
    Cs, Ts = oracle(p, rows=rows)
    assert np.array_equal(Cs, C[rows]) and np.array_equal(Ts, T[rows])
    with pytest.raises(ValueError):
        oracle(p, rows=np.array([p.m], dtype=np.int64))


def test_stored_order_accumulation_is_sequential_fp64():
    # 1e16 + 1 - 1e16 in stored order gives 0 in fp64 (the 1 is absorbed); a reordered or
    # pairwise sum would give 1.  Pins "accumulate in stored order".
    B = np.array([[1.0], [1.0], [1.0]], dtype=np.float32)
    vals = np.array([1e16, 1.0, -1e16], dtype=np.float32)
    big = np.float64(np.float32(1e16))
    C, _ = spmm_csr_oracle(1, 1, np.array([0, 3], np.int32), np.array([0, 1, 2], np.int32), vals, B)
    assert C[0, 0] == (big + 1.0) - big


def test_bias_activation_layer_oracle():
    # hand-worked on the 3x3 fixture: A.B = [[11 14],[0 0],[9 12]]; bias [-10, 1] -> [[1 15],[-10 1],[-1 13]];
    # ReLU -> [[1 15],[0 1],[0 13]]
    g = read_fixture("handworked_3x3.txt")
    bias = np.array([-10.0, 1.0], dtype=np.float32)
    C, T = spmm_bias_act_oracle(g["m"], g["n"], g["rowptr"], g["colidx"], g["vals"], g["B"], bias, relu=False)
    assert np.array_equal(C, np.array([[1, 15], [-10, 1], [-1, 13]], dtype=np.float64))
    assert np.array_equal(T, g["T"] + np.array([10.0, 1.0]))
    C, _ = spmm_bias_act_oracle(g["m"], g["n"], g["rowptr"], g["colidx"], g["vals"], g["B"], bias, relu=True)
    assert np.array_equal(C, np.array([[1, 15], [0, 1], [0, 13]], dtype=np.float64))
    # no bias, no activation: the plain product; dense cross-check with numpy on a random pattern
    p = csr_from_row_lengths([4, 0, 9, 2, 6], 12, 7, seed=21)
    b = np.random.default_rng(1).standard_normal(7).astype(np.float32)
    C0, T0 = oracle(p)
    C1, T1 = spmm_bias_act_oracle(p.m, p.n, p.rowptr, p.colidx, p.vals, p.B, None, relu=False)
    assert np.array_equal(C0, C1) and np.array_equal(T0, T1)
    C2, _ = spmm_bias_act_oracle(p.m, p.n, p.rowptr, p.colidx, p.vals, p.B, b, relu=True)
    ref = np.maximum(densify(p) @ p.B[:, :p.n].astype(np.float64) + b.astype(np.float64), 0.0)
    assert np.all(np.abs(C2 - ref) <= 1e-12 * (T0 + 1)) and np.all(C2 >= 0) and np.array_equal(C2[1], np.maximum(b.astype(np.float64), 0))
