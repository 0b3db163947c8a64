"""Randomised pins of the two fp64 oracles (hypothesis; runs without a GPU).

Arbitrary small CSR patterns, drawn entry by entry (so rows may repeat a column, be unsorted or be empty), with
small-integer values: the oracle must equal an exact integer evaluation of the definition written with Python
integers and explicit loops over (row, stored entry, column) -- a different arithmetic type and a different code
path from the C oracle.  SpMM: C_ik = sum_j A_ij B_jk (paper, Section 4.2); SDDMM: D_ij = A_ij sum_t B_it C_tj on
the stored entries (paper, Section 3.1).
"""
import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import sddmm_csr_oracle, spmm_csr_oracle


@st.composite
def csr_problem(draw):
    m = draw(st.integers(1, 7))
    k = draw(st.integers(1, 7))
    n = draw(st.integers(1, 6))
    pad = draw(st.integers(0, 3))
    lens = [draw(st.integers(0, 2 * k)) for _ in range(m)]
    cols = [draw(st.integers(0, k - 1)) for _ in range(sum(lens))]
    vals = [draw(st.integers(-4, 4)) for _ in range(sum(lens))]
    B = [[draw(st.integers(-8, 8)) for _ in range(n)] for _ in range(k)]
    return m, k, n, pad, lens, cols, vals, B


@settings(max_examples=150, deadline=None)
@given(csr_problem())
def test_spmm_oracle_equals_integer_definition(prob):
    m, k, n, pad, lens, cols, vals, B = prob
    rowptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ldb = n + pad
    Bp = np.full((k, ldb), np.nan, dtype=np.float32)
    Bp[:, :n] = np.array(B, dtype=np.float32).reshape(k, n)
    C, T = spmm_csr_oracle(m, n, rowptr, np.array(cols, dtype=np.int32), np.array(vals, dtype=np.float32), Bp, ldb)
    p = 0
    for i in range(m):
        exact = [0] * n
        mag = [0] * n
        for _ in range(lens[i]):
            for c in range(n):
                exact[c] += vals[p] * B[cols[p]][c]
                mag[c] += abs(vals[p]) * abs(B[cols[p]][c])
            p += 1
        assert [int(x) for x in C[i]] == exact and all(float(x).is_integer() for x in C[i])
        assert [int(x) for x in T[i]] == mag


@settings(max_examples=150, deadline=None)
@given(csr_problem(), st.integers(1, 5))
def test_sddmm_oracle_equals_integer_definition(prob, d):
    m, k, _, pad, lens, cols, vals, _ = prob
    rng = np.random.default_rng(m * 100 + k * 10 + d)
    X = rng.integers(-8, 9, size=(m, d))
    Y = rng.integers(-8, 9, size=(k, d))  # Y = C^T: row j is column j of C
    rowptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ld = d + pad
    Xp = np.full((m, ld), np.nan, dtype=np.float32)
    Xp[:, :d] = X
    Yp = np.full((k, ld), np.nan, dtype=np.float32)
    Yp[:, :d] = Y
    out, _ = sddmm_csr_oracle(m, d, rowptr, np.array(cols, dtype=np.int32), np.array(vals, dtype=np.float32), Xp, Yp)
    p = 0
    for i in range(m):
        for _ in range(lens[i]):
            exact = vals[p] * sum(int(X[i][t]) * int(Y[cols[p]][t]) for t in range(d))
            assert float(out[p]) == float(exact)
            p += 1
