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
    for rep in range(6 if cfg == 4 else 25):  # double-buffered panels / hot-cold loads: the same bits every time
        C2 = d.run_planned(plan)
        assert np.array_equal(C, C2), f"repeated planned run {rep} differs"
    del C2
    if cfg == 4:
        info = plan.info()
        assert info.n_hot_columns > 0 and 0.3 < info.hot_share < 0.8  # B exceeds the memory-side cache: hot/cold split
        with tuning("hot=0"):
            plan0 = d.make_plan()
            assert plan0.info().n_hot_columns == 0
            assert np.array_equal(C, d.run_planned(plan0)), "hot/cold split changed the result"
            plan0.destroy()
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


def test_operands_beyond_two_to_the_31_elements():
    """B and C with more than 2^31 elements each (64-bit addressing inside the kernels): m = k = 2^22 + 5, n = 520.
    B is drawn on the device; the oracle sees a compact copy of the B rows that the sampled rows of A reference."""
    from oracle import spmm_csr_oracle

    dev = torch.device("cuda:0")
    m = k = (1 << 22) + 5
    n = 520
    assert m * n > 2**31
    rng = np.random.default_rng(31)
    lens = np.full(m, 3, dtype=np.int64)
    lens[rng.integers(0, m, size=1000)] = 0
    lens[m - 2] = 3000  # a long row whose C row lies beyond element 2^31
    lens[7] = 700
    rowptr = np.zeros(m + 1, dtype=np.int64)
    np.cumsum(lens, out=rowptr[1:])
    nnz = int(rowptr[-1])
    colidx = rng.integers(0, k, size=nnz, dtype=np.int64)
    colidx[::5] = k - 1 - (colidx[::5] % 1000)  # many references to the last rows of B (beyond element 2^31)
    vals = rng.uniform(-1, 1, size=nnz).astype(np.float32)
    g = torch.Generator(device=dev).manual_seed(5)
    B = torch.randn((k, n), generator=g, dtype=torch.float32, device=dev)
    C = torch.full((m, n), -9.0, dtype=torch.float32, device=dev)
    rp_d = torch.from_numpy(rowptr.astype(np.int32)).to(dev)
    ci_d = torch.from_numpy(colidx.astype(np.int32)).to(dev)
    va_d = torch.from_numpy(vals).to(dev)
    rows = np.unique(np.concatenate([[0, 7, m - 2, m - 1], rng.integers(m - 100000, m, size=150),
                                     rng.integers(0, m, size=150), np.nonzero(lens == 0)[0][:10]]))

    def check(label):
        torch.cuda.synchronize()
        # compact problem for the oracle: only the sampled rows and the B rows they touch
        seg = [np.arange(rowptr[i], rowptr[i + 1]) for i in rows]
        idx = np.concatenate(seg)
        cols, inv = np.unique(colidx[idx], return_inverse=True)
        Bsub = B[torch.from_numpy(cols).to(dev)].cpu().numpy()
        rp = np.concatenate([[0], np.cumsum([len(s) for s in seg])]).astype(np.int32)
        C_ref, T = spmm_csr_oracle(len(rows), n, rp, inv.astype(np.int32), vals[idx], Bsub)
        got = C[torch.from_numpy(rows).to(dev)].cpu().numpy().astype(np.float64)
        bad = ~(np.abs(got - C_ref) <= RTOL_T * T + ATOL)
        assert not bad.any(), f"{label}: {int(bad.sum())} sampled elements out of tolerance"

    plan = sp.scorch_spmm_plan(m, k, n, rp_d, nnz, colidx=ci_d)
    sp.scorch_spmm_csr_planned(plan, rp_d, ci_d, va_d, B, C)
    check("planned")
    plan.destroy()
    C.fill_(-9.0)
    sp.scorch_spmm_csr(m, k, n, rp_d, ci_d, va_d, B, C)
    check("plan-free")
