"""Seeded generators: determinism, CSR validity, and the statistics each workload is meant to have."""
import numpy as np
import pytest

from workloads import (chung_lu_graph, count_unique_columns, csr_from_row_lengths, integer_valued,
                       make_scaled_config, min_traffic_bytes, pruned_weight, tiny_powerlaw, uniform_rows)


def rows_sorted_unique(p):
    d = np.diff(p.colidx.astype(np.int64))
    interior = np.ones(p.nnz - 1, dtype=bool)
    ends = p.rowptr[1:-1].astype(np.int64)
    ends = ends[(ends > 0) & (ends < p.nnz)]
    interior[ends - 1] = False
    return bool(np.all(d[interior] > 0))


@pytest.mark.parametrize("cfg,scale", [(1, 1.0), (2, 0.05), (3, 0.05), (4, 0.004), (5, 0.05)])
def test_configs_valid_and_deterministic(cfg, scale):
    a = make_scaled_config(cfg, scale, seed=0)
    b = make_scaled_config(cfg, scale, seed=0)
    c = make_scaled_config(cfg, scale, seed=1)
    a.check()
    assert rows_sorted_unique(a)
    for x, y in ((a.rowptr, b.rowptr), (a.colidx, b.colidx), (a.vals, b.vals), (a.B, b.B)):
        assert np.array_equal(x, y)
    assert not np.array_equal(a.B, c.B)
    assert min_traffic_bytes(a) == a.nnz * 8 + (a.m + 1) * 4 + a.m * a.n * 4 + count_unique_columns(a) * a.n * 4


def test_config1_shape_and_values():
    p = tiny_powerlaw()
    assert (p.m, p.k, p.n) == (4096, 4096, 64)
    assert 14000 < p.nnz < 18500
    L = p.row_lengths
    assert L.min() >= 2 and L.max() <= 65  # >= 1 target + self-loop
    rows = np.repeat(np.arange(p.m), L)
    assert np.all(np.isin(np.arange(p.m), p.colidx[rows == p.colidx]))  # every row stores its diagonal
    expect = (1.0 / np.sqrt(L[rows].astype(np.float64) * L[p.colidx])).astype(np.float32)
    assert np.array_equal(p.vals, expect)


def test_config2_fixed_row_length():
    p = uniform_rows(m=512, k=16384, density=0.01, n=8, seed=3)
    assert np.all(p.row_lengths == 164)
    assert rows_sorted_unique(p)
    assert np.abs(p.vals).max() <= 1.0 and abs(float(p.vals.mean())) < 0.02
    # columns uniform: mean near k/2
    assert abs(p.colidx.mean() / 16384 - 0.5) < 0.02


def test_chung_lu_symmetric_and_normalised():
    p = chung_lu_graph(3000, 14.0, 400.0, 2.1, 4, normalize="sym", self_loops=True, seed=2)
    rows = np.repeat(np.arange(p.m), p.row_lengths)
    fwd = set(zip(rows.tolist(), p.colidx.tolist()))
    assert all((c, r) in fwd for r, c in fwd)  # symmetric pattern
    assert all((i, i) in fwd for i in range(p.m))
    L = p.row_lengths
    assert L.max() > 20 * np.median(L)  # skewed degrees
    q = chung_lu_graph(3000, 14.0, 400.0, 2.1, 4, normalize="row", self_loops=False, seed=2)
    sums = np.zeros(q.m)
    np.add.at(sums, np.repeat(np.arange(q.m), q.row_lengths), q.vals.astype(np.float64))
    nz = q.row_lengths > 0
    assert np.allclose(sums[nz], 1.0, atol=1e-5)
    # relabelling decorrelates degree from index
    r = np.corrcoef(np.arange(p.m), L)[0, 1]
    assert abs(r) < 0.1


def test_pruned_weight_density():
    p = pruned_weight(m=128, k=4096, sparsity=0.9, n=16, seed=5)
    assert abs(p.nnz / (128 * 4096) - 0.1) < 0.005
    assert abs(float(p.vals.std()) - 0.02) < 0.002


def test_integer_valued_keeps_pattern():
    p = csr_from_row_lengths([5, 0, 9], 20, 6, seed=1, ldb=8)
    q = integer_valued(p, seed=2)
    assert np.array_equal(p.rowptr, q.rowptr) and np.array_equal(p.colidx, q.colidx)
    assert set(np.unique(q.vals)).issubset({-4., -3., -2., -1., 1., 2., 3., 4.})
    assert np.all(np.abs(q.B[:, :6]) <= 8) and np.all(q.B[:, :6] == np.round(q.B[:, :6]))
    assert np.all(np.isnan(q.B[:, 6:]))
