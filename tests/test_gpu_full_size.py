"""GPU parity at the full sizes of the five workloads, in the configuration bench.py times (default plan).

Workloads 1-3: every element against the oracle.  Workloads 4 and 5: sampled rows against the oracle (heaviest
rows, empty rows, a seeded random sample), plus, for every row, the row-sum property
    sum_c C[i,c] = sum_p vals[p] * (B.1)[colidx[p]]
checked in fp64 against the summed per-element tolerance, which holds at any size.
"""
import os

import numpy as np
import pytest
import torch

import paper_2405_16883_amd as sp
from workloads import integer_valued, make_config

from gpu_util import ATOL, RTOL_T, DeviceProblem, check_against_oracle, tuning

pytestmark = pytest.mark.gpu
CACHE = os.environ.get("SCORCH_WORKLOAD_CACHE")


def sample_rows(p, count, seed):
    L = p.row_lengths
    heavy = np.argsort(L)[-40:]
    empty = np.nonzero(L == 0)[0][:40]
    rnd = np.random.default_rng(seed).choice(p.m, size=min(count, p.m), replace=False)
    edge = np.array([0, p.m - 1])
    return np.unique(np.concatenate([heavy, empty, rnd, edge])).astype(np.int64)


def row_sum_property(p, C):
    """|sum_c C[i,c] - A.(B.1)| <= sum_c (RTOL_T * T[i,c] + ATOL), all rows, in fp64 with numpy only."""
    rows = np.repeat(np.arange(p.m), p.row_lengths)
    Bn = p.B[:, :p.n].astype(np.float64)
    b1 = Bn.sum(axis=1)
    babs = np.abs(Bn).sum(axis=1)
    v = p.vals.astype(np.float64)
    rhs = np.bincount(rows, weights=v * b1[p.colidx], minlength=p.m)
    tsum = np.bincount(rows, weights=np.abs(v) * babs[p.colidx], minlength=p.m)
    lhs = C.astype(np.float64).sum(axis=1)
    bound = RTOL_T * tsum + ATOL * p.n + 1e-12 * tsum
    bad = ~(np.abs(lhs - rhs) <= bound)
    assert not bad.any(), f"row-sum property fails on {int(bad.sum())} rows, first {np.nonzero(bad)[0][:5]}"


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_full_size_every_element(cfg):
    p = make_config(cfg, seed=0, cache_dir=CACHE)
    print(f"workload {cfg}: m={p.m} n={p.n} nnz={p.nnz}", flush=True)
    d = DeviceProblem(p)
    plan = d.make_plan()
    check_against_oracle(p, d.run_planned(plan), d.ldc, label=f"workload {cfg} planned")
    check_against_oracle(p, d.run_natural(), d.ldc, label=f"workload {cfg} plan-free")
    plan.destroy()
    q = integer_valued(p, seed=3)
    d = DeviceProblem(q)
    plan = d.make_plan()
    check_against_oracle(q, d.run_planned(plan), d.ldc, exact=True, label=f"workload {cfg} planned int")
    plan.destroy()


@pytest.mark.parametrize("cfg", [5, 4])
def test_full_size_sampled_rows_and_row_sums(cfg):
    p = make_config(cfg, seed=0, cache_dir=CACHE)
    print(f"workload {cfg}: m={p.m} n={p.n} nnz={p.nnz}", flush=True)
    rows = sample_rows(p, 1500 if cfg == 4 else 150, seed=cfg)
    d = DeviceProblem(p)
    plan = d.make_plan()
    C = d.run_planned(plan)
    check_against_oracle(p, C, d.ldc, rows=rows, label=f"workload {cfg} planned, {len(rows)} sampled rows")
    row_sum_property(p, C[:p.m, :p.n])
    C2 = d.run_planned(plan)
    assert np.array_equal(C, C2), "repeated planned runs differ"
    del C2
    Cn = d.run_natural()
    check_against_oracle(p, Cn, d.ldc, rows=rows, label=f"workload {cfg} plan-free, sampled rows")
    del Cn, C
    assert plan.info().mode == (2 if cfg == 5 else 0)  # workload 5 runs the panel kernel by default
    plan.destroy()
    if cfg == 5:
        with tuning("panel=0"):  # the XCD-sliced gather kernel (with the packed copy of B) on the same workload
            plan = d.make_plan()
            assert plan.info().mode == 1
            check_against_oracle(p, d.run_planned(plan), d.ldc, rows=rows, label="workload 5 sliced gather, sampled rows")
            plan.destroy()
    # integer twin: bit-exact on the sampled rows
    q = integer_valued(p, seed=4)
    d.Bfull.copy_(torch.from_numpy(q.B))
    d.vals.copy_(torch.from_numpy(q.vals))
    d.p = q
    plan = d.make_plan()
    check_against_oracle(q, d.run_planned(plan), d.ldc, exact=True, rows=rows, label=f"workload {cfg} planned int")
    plan.destroy()
