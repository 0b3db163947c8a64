"""GPU parity of the fused bias + activation epilogue: C = act(A.B + bias) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2405_16883_amd as sp
from oracle import spmm_bias_act_oracle
from workloads import csr_from_row_lengths, integer_valued, make_config, make_scaled_config

from gpu_util import ATOL, RTOL_T, DeviceProblem, tuning

pytestmark = pytest.mark.gpu


def run_epilogue(p, bias, relu, exact=False, label="", tune=None):
    with tuning(tune):
        d = DeviceProblem(p)
        plan = d.make_plan()
        d.reset_C()
        bias_d = torch.from_numpy(bias).to(d.dev) if bias is not None else None
        sp.scorch_spmm_csr_planned_epilogue(plan, d.rowptr, d.colidx, d.vals, d._B_arg(), bias_d,
                                            sp.ACT_RELU if relu else sp.ACT_IDENTITY, d._C_arg())
        torch.cuda.synchronize()
        C = d.Cfull.cpu().numpy()[:p.m, :p.n].astype(np.float64)
        plain = None
        if bias is None and not relu:
            plain = d.run_planned(plan)[:p.m, :p.n].astype(np.float64)
        plan.destroy()
    C_ref, T = spmm_bias_act_oracle(p.m, p.n, p.rowptr, p.colidx, p.vals, p.B, bias, relu, p.ldb)
    if exact:
        assert np.array_equal(C, C_ref), f"{label}: differs from the exact integer result"
    else:
        bad = ~(np.abs(C - C_ref) <= RTOL_T * T + ATOL)
        assert not bad.any(), f"{label}: {int(bad.sum())} elements out of tolerance"
    if plain is not None:
        assert np.array_equal(C, plain), f"{label}: identity epilogue differs from the plain call"


TUNES = [None, "bn=64,alpha=2,lw=8,ch=32,bch=64", "sliced=1,pack=1", "panel=1", "panel=2", "panel=0",
         "bn=64,alpha=2,lw=8,ch=32,bch=64,fix=1"]


@pytest.mark.parametrize("tune", TUNES)
@pytest.mark.parametrize("cfg,scale", [(3, 0.08), (4, 0.006), (5, 0.06)])
def test_epilogue_on_small_workloads(cfg, scale, tune):
    p = make_scaled_config(cfg, scale, seed=9)
    rng = np.random.default_rng(cfg)
    bias = rng.standard_normal(p.n).astype(np.float32)
    for b, relu in ((bias, True), (bias, False), (None, True), (None, False)):
        run_epilogue(p, b, relu, label=f"{p.name} bias={b is not None} relu={relu} [{tune}]", tune=tune)
    q = integer_valued(p, seed=3)
    ibias = rng.integers(-20, 21, size=p.n).astype(np.float32)
    run_epilogue(q, ibias, True, exact=True, label=f"{p.name} int [{tune}]", tune=tune)


@pytest.mark.parametrize("n", [1, 3, 4, 64, 100, 130, 300])
def test_epilogue_column_counts_and_split_rows(n):
    rng = np.random.default_rng(n)
    lens = np.concatenate([rng.integers(0, 40, size=120), [3000, 0, 300, 65, 1]])
    p = integer_valued(csr_from_row_lengths(lens, 500, n, seed=n, duplicates=True), seed=n)
    bias = rng.integers(-50, 51, size=n).astype(np.float32)
    run_epilogue(p, bias, True, exact=True, label=f"n={n}", tune="ch=128,bch=256")
    run_epilogue(p, bias, False, exact=True, label=f"n={n} no act", tune="ch=128,bch=256")


@pytest.mark.parametrize("tune", [None, "bn=256,lw=64", "bn=256,lw=32,ch=64", "bn=128,lw=8"])
@pytest.mark.parametrize("n", [1, 2, 4])
def test_one_lane_groups_split_the_entries_of_a_window(n, tune):
    """n <= 4: the lanes of a wavefront take the entries of a window and each row's lane adds up its products.
    Many short rows of every length up to the window limit, medium rows in between (their entries lie inside the
    staged span but belong to another path), empty rows, one long row; with and without bias and ReLU."""
    rng = np.random.default_rng(7 * n)
    lens = rng.integers(0, 66, size=3000)
    lens[rng.integers(0, 3000, size=200)] = 0
    lens[rng.integers(0, 3000, size=40)] = rng.integers(65, 300, size=40)
    lens[1234] = 5000
    p = csr_from_row_lengths(lens, 6000, n, seed=n, duplicates=False)
    bias = rng.standard_normal(n).astype(np.float32)
    run_epilogue(p, None, False, label=f"n={n} plain [{tune}]", tune=tune)
    run_epilogue(p, bias, True, label=f"n={n} bias relu [{tune}]", tune=tune)
    q = integer_valued(p, seed=n)
    run_epilogue(q, rng.integers(-9, 10, size=n).astype(np.float32), True, exact=True, label=f"n={n} int [{tune}]", tune=tune)


def test_epilogue_full_size_gcn_layer():
    p = make_config(3, seed=0)
    bias = np.random.default_rng(2).standard_normal(p.n).astype(np.float32) * 0.1
    run_epilogue(p, bias, True, label="workload 3 bias+relu")


def test_epilogue_rejects_unknown_activation():
    p = make_scaled_config(1, 0.2, seed=1)
    d = DeviceProblem(p)
    plan = d.make_plan()
    with pytest.raises(sp.ScorchError) as e:
        sp.scorch_spmm_csr_planned_epilogue(plan, d.rowptr, d.colidx, d.vals, d._B_arg(), None, 7, d._C_arg())
    assert e.value.status == sp.binding.SCORCH_ERR_INVALID_ARG
    plan.destroy()
