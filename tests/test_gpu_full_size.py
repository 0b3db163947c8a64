"""GPU parity at the full sizes of the five workloads, in the configuration bench.py times (default plan).

All five workloads: every element against the oracle (for workloads 4 and 5 the oracle runs over contiguous blocks of
rows on all host cores, see gpu_util.check_every_row_chunked), planned and plan-free, plus the integer-valued twin bit
for bit.  Workloads 4 and 5 additionally check, for every row, the row-sum property
    sum_c C[i,c] = sum_p vals[p] * (B.1)[colidx[p]]
in fp64 against the summed per-element tolerance.
"""
import os

import numpy as np
import pytest
import torch

import paper_2405_16883_amd as sp
from workloads import integer_valued, make_config

from gpu_util import ATOL, RTOL_T, DeviceProblem, check_against_oracle, check_every_row_chunked, tuning

pytestmark = pytest.mark.gpu
CACHE = os.environ.get("SCORCH_WORKLOAD_CACHE")


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
def test_full_size_every_element_large_workloads(cfg):
    """Workloads 4 (the benchmark's headline) and 5 (panel kernel): EVERY element of the planned result (default plan:
    hot/cold gathers / LDS panels), of the plan-free result and, for workload 5, of the XCD-sliced gather, against the
    oracle, which runs over all rows in contiguous blocks spread over the host cores.  Then the integer-valued twin,
    bit for bit on every element.  The row-sum property stays as an extra."""
    p = make_config(cfg, seed=0, cache_dir=CACHE)
    print(f"workload {cfg}: m={p.m} n={p.n} nnz={p.nnz}", flush=True)
    d = DeviceProblem(p)
    plan = d.make_plan()
    C = d.run_planned(plan)
    outputs = {f"workload {cfg} planned": C}
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
    assert plan.info().mode == (2 if cfg == 5 else 0)  # workload 5 runs the panel kernel by default
    plan.destroy()
    outputs[f"workload {cfg} plan-free"] = d.run_natural()
    if cfg == 5:
        with tuning("panel=0"):  # the XCD-sliced gather kernel (with the packed copy of B) on the same workload
            plan = d.make_plan()
            assert plan.info().mode == 1
            outputs["workload 5 sliced gather"] = d.run_planned(plan)
            plan.destroy()
    print("oracle over all rows ...", flush=True)
    worst = check_every_row_chunked(p, outputs)
    print("worst err/bound:", {k: round(v, 4) for k, v in worst.items()}, flush=True)
    del outputs, C
    # integer twin: bit-exact on every element
    q = integer_valued(p, seed=4)
    d.Bfull.copy_(torch.from_numpy(q.B))
    d.vals.copy_(torch.from_numpy(q.vals))
    d.p = q
    plan = d.make_plan()
    outputs = {f"workload {cfg} planned int": d.run_planned(plan)}
    plan.destroy()
    outputs[f"workload {cfg} plan-free int"] = d.run_natural()
    check_every_row_chunked(q, outputs, exact=True)


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
