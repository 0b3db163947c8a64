"""GPU parity of SDDMM (D = A (.) (B C) on the stored entries) against the fp64 oracle, through the C ABI.

Bar: bit-exact on small-integer inputs; |D - D_ref| <= 1e-5 * |A_ij| sum_t |B_it||C_tj| + 1e-7 on fp32 inputs.
"""
import numpy as np
import pytest
import torch

import paper_2405_16883_amd as sp
from oracle import sddmm_csr_oracle
from workloads import csr_from_row_lengths, integer_valued, make_config, make_scaled_config

from gpu_util import ATOL, RTOL_T, tuning

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def factors(m, k, d, seed, integer=False, ldb=None, ldct=None):
    rng = np.random.default_rng(seed)
    ldb = ldb or d
    ldct = ldct or d
    B = np.full((m, ldb), np.nan, np.float32)
    Ct = np.full((k, ldct), np.nan, np.float32)
    if integer:
        B[:, :d] = rng.integers(-8, 9, size=(m, d))
        Ct[:, :d] = rng.integers(-8, 9, size=(k, d))
    else:
        B[:, :d] = rng.standard_normal((m, d))
        Ct[:, :d] = rng.standard_normal((k, d))
    return B, Ct


def run_and_check(p, d, seed, integer=False, ldb=None, ldct=None, label="", planned=True, in_place=False):
    B, Ct = factors(p.m, p.k, d, seed, integer, ldb, ldct)
    D_ref, T = sddmm_csr_oracle(p.m, d, p.rowptr, p.colidx, p.vals, B, Ct)
    rowptr = torch.from_numpy(p.rowptr).to(DEV)
    colidx = torch.from_numpy(p.colidx).to(DEV) if p.nnz else torch.zeros(0, dtype=torch.int32, device=DEV)
    vals = torch.from_numpy(p.vals).to(DEV) if p.nnz else torch.zeros(0, dtype=torch.float32, device=DEV)
    Bd = torch.from_numpy(B).to(DEV).as_strided((p.m, d), (B.shape[1], 1))
    Cd = torch.from_numpy(Ct).to(DEV).as_strided((p.k, d), (Ct.shape[1], 1))
    out = vals if in_place else torch.full((max(p.nnz, 1),), -77.0, dtype=torch.float32, device=DEV)
    if planned:
        plan = sp.scorch_spmm_plan(p.m, p.k, p.n, rowptr, p.nnz, colidx=colidx)
        sp.scorch_sddmm_csr_planned(plan, d, rowptr, colidx, vals, Bd, Cd, out)
        torch.cuda.synchronize()
        plan.destroy()
    else:
        sp.scorch_sddmm_csr(p.m, p.k, d, rowptr, colidx, vals, Bd, Cd, out)
        torch.cuda.synchronize()
    D = out.cpu().numpy()[:p.nnz].astype(np.float64)
    if integer:
        bad = D != D_ref
        assert not bad.any(), f"{label}: {int(bad.sum())} entries differ from the exact integer result, first {np.nonzero(bad)[0][:4]}"
    else:
        err = np.abs(D - D_ref)
        bound = RTOL_T * T + ATOL
        bad = ~(err <= bound)
        assert not bad.any(), f"{label}: {int(bad.sum())} entries out of tolerance, worst {np.nanmax(err / bound):.3g} at {np.nonzero(bad)[0][:4]}"


TUNES = [None, "bn=64,alpha=2,lw=8,ch=32,bch=64", "bn=256,lw=64,ch=256,bch=256", "bn=128,lw=0,ch=64,bch=128",
         "sdblk=1", "sdblk=3"]  # sdblk: entries dealt to the XCDs by column block (1 or 3 blocks per XCD)


@pytest.mark.parametrize("tune", TUNES)
@pytest.mark.parametrize("cfg,scale", [(1, 1.0), (3, 0.08), (4, 0.006), (2, 0.12)])
def test_sddmm_small_workloads(cfg, scale, tune):
    with tuning(tune):
        p = make_scaled_config(cfg, scale, seed=7)
        d = 128 if cfg != 1 else 64
        run_and_check(p, d, 1, label=f"{p.name} d={d} [{tune}]")
        run_and_check(integer_valued(p, seed=2), d, 2, integer=True, label=f"{p.name} int d={d} [{tune}]")
        run_and_check(p, d, 3, planned=False, label=f"{p.name} plan-free d={d}")


@pytest.mark.parametrize("d", [1, 2, 3, 4, 5, 7, 8, 31, 32, 33, 64, 100, 128, 130, 255, 256, 257, 260, 301, 512, 516, 1000, 1001, 1023, 1024])
def test_sddmm_inner_dimensions(d):
    rng = np.random.default_rng(d)
    lens = np.concatenate([rng.integers(0, 40, size=150), [700, 0, 300, 65, 64, 33, 32, 1, 9, 8, 7]])
    p = csr_from_row_lengths(lens, 500, 4, seed=d, duplicates=True, sorted_cols=False)
    with tuning("ch=128,bch=256"):
        run_and_check(p, d, d, label=f"d={d}")
        run_and_check(integer_valued(p, seed=d), d, d + 1, integer=True, label=f"d={d} int")
        run_and_check(integer_valued(p, seed=d), d, d + 2, integer=True, planned=False, label=f"d={d} int plan-free")
    with tuning("sdblk=2"):  # column blocks over the XCDs
        run_and_check(p, d, d, label=f"d={d} column blocks")
        run_and_check(integer_valued(p, seed=d), d, d + 1, integer=True, label=f"d={d} int column blocks")


@pytest.mark.parametrize("d,ldb,ldct", [(64, 72, 68), (100, 101, 103), (7, 9, 8), (128, 132, 136), (256, 260, 256), (300, 301, 303),
                                        (1021, 1024, 1022)])
def test_sddmm_leading_dimensions(d, ldb, ldct):
    p = csr_from_row_lengths(np.random.default_rng(3).integers(0, 90, size=300), 400, 4, seed=3)
    run_and_check(p, d, 5, ldb=ldb, ldct=ldct, label=f"d={d} ldb={ldb} ldct={ldct}")  # padding holds NaN
    run_and_check(integer_valued(p, seed=4), d, 6, integer=True, ldb=ldb, ldct=ldct, label=f"d={d} padded int")


def test_sddmm_edge_patterns_and_in_place():
    for lens in ([0] * 300, [5], [0, 0, 5000, 0], [20000], [33] * 100 + [0], [1] * 1000):
        p = integer_valued(csr_from_row_lengths(lens, 3000, 4, seed=8, duplicates=True), seed=8)
        run_and_check(p, 64, 9, integer=True, label=f"lens={lens[:3]}..")
        run_and_check(p, 64, 9, integer=True, planned=False, label=f"lens={lens[:3]}.. plan-free")
        run_and_check(p, 64, 9, integer=True, in_place=True, label=f"lens={lens[:3]}.. in place")
        with tuning("sdblk=1"):
            run_and_check(p, 64, 9, integer=True, label=f"lens={lens[:3]}.. column blocks")
            run_and_check(p, 64, 9, integer=True, in_place=True, label=f"lens={lens[:3]}.. column blocks in place")


def test_sddmm_argument_errors():
    lib = sp.load_library()
    z = torch.zeros(8, dtype=torch.int32, device=DEV)
    f = torch.zeros((4, 2048), dtype=torch.float32, device=DEV)
    st = lib.scorch_sddmm_csr(4, 4, 2048, z.data_ptr(), z.data_ptr(), f.data_ptr(), f.data_ptr(), 2048, f.data_ptr(), 2048, f.data_ptr(), None)
    assert st == sp.binding.SCORCH_ERR_UNSUPPORTED  # d > 1024
    st = lib.scorch_sddmm_csr(4, 4, 8, z.data_ptr(), z.data_ptr(), f.data_ptr(), f.data_ptr(), 4, f.data_ptr(), 8, f.data_ptr(), None)
    assert st == sp.binding.SCORCH_ERR_INVALID_ARG  # ldb < d
    st = lib.scorch_sddmm_csr(0, 4, 8, None, None, None, None, 8, None, 8, None, None)
    assert st == 0  # m = 0: nothing to do


def test_sddmm_full_size_gcn_graph():
    p = make_config(3, seed=0)
    run_and_check(p, 128, 11, label="workload 3 pattern, d=128")
    run_and_check(integer_valued(p, seed=5), 128, 12, integer=True, label="workload 3 pattern int")


def test_sddmm_full_size_uniform_pattern_uses_column_blocks():
    """Workload 2's pattern with d = 256: the second factor is 17 MB, rows have 164 entries, so the planned call deals
    the entries to the XCDs by column block (its default there); every entry against the oracle."""
    p = make_config(2, seed=0)
    run_and_check(p, 256, 13, label="workload 2 pattern, d=256")
    run_and_check(integer_valued(p, seed=6), 256, 14, integer=True, label="workload 2 pattern int, d=256")


@pytest.mark.parametrize("block", range(6))
def test_sddmm_random_small_problems(block):
    """Seeded random shapes, row-length mixes, leading dimensions and forced plan parameters."""
    for i in range(block * 15, block * 15 + 15):
        rng = np.random.default_rng(5000 + i)
        m = int(rng.choice([1, 3, 17, 64, 65, 130, 300]))
        k = int(rng.choice([1, 2, 31, 33, 100, 700, 2500]))
        d = int(rng.choice([1, 2, 3, 4, 5, 8, 31, 32, 33, 64, 65, 100, 127, 128, 129, 256, 257, 300, 513, 1000, 1023]))
        kind = int(rng.integers(0, 3))
        if kind == 0:
            lens = rng.integers(0, min(k, 40) + 1, size=m)
        elif kind == 1:
            lens = np.minimum((rng.pareto(1.2, size=m) * 3).astype(np.int64), 3 * k)
        else:
            lens = np.zeros(m, dtype=np.int64)
            lens[rng.integers(0, m, size=max(1, m // 8))] = int(rng.integers(1, 2000))
        dup = bool(rng.integers(0, 2)) or int(lens.max(initial=0)) > k
        p = csr_from_row_lengths(lens, k, 4, seed=i, duplicates=dup, sorted_cols=bool(rng.integers(0, 2)))
        ldb = d + int(rng.choice([0, 0, 1, 3, 4]))
        ldct = d + int(rng.choice([0, 0, 1, 2, 4]))
        tune = TUNES[int(rng.integers(0, len(TUNES)))]
        label = f"case {i}: m={m} k={k} d={d} nnz={p.nnz} ldb={ldb} ldct={ldct} [{tune}]"
        print(label, flush=True)
        with tuning(tune):
            run_and_check(p, d, i, ldb=ldb, ldct=ldct, label=label)
            run_and_check(integer_valued(p, seed=i), d, i + 1, integer=True, ldb=ldb, ldct=ldct, label=label + " int")
            run_and_check(integer_valued(p, seed=i), d, i + 2, integer=True, ldb=ldb, ldct=ldct, planned=False,
                          label=label + " int plan-free")


@pytest.mark.parametrize("m,d", [(16384 + 37, 128), (16384 + 37, 300), (16384 + 37, 33), (65536 + 5, 8), (65536 + 5, 32)])
def test_sddmm_plan_free_row_runs(m, d):
    """The plan-free kernel gives a wavefront a run of consecutive rows (4 with 16 384 rows or more, up to 16 with
    65 536 rows or more and narrow lane groups): row lengths sit on every staging and long-row limit, in runs that mix
    them, in a matrix whose last workgroup is ragged."""
    rng = np.random.default_rng(31)
    lens = rng.integers(0, 41, size=m)
    special = [0, 1, 31, 32, 33, 64, 255, 256, 257, 287, 288, 289, 319, 320, 321, 2047, 2048, 2049, 3000]
    for i, pos in enumerate(range(5, m - 64, 211)):
        lens[pos] = special[i % len(special)]
    lens[1000:1016] = 20
    lens[2000:2004] = [80, 80, 80, 80]
    lens[3000:3016] = 300  # a workgroup with many rows beyond 256 entries: every wavefront keeps its own
    lens[4000:4016] = [0] * 15 + [257]  # a single such row in a workgroup: shared by the 4 wavefronts
    lens[m - 3:] = [2049, 0, 33]
    p = csr_from_row_lengths(lens.tolist(), 5000, 4, seed=32, duplicates=True, sorted_cols=False)
    run_and_check(p, d, 5, planned=False, label=f"plan-free row runs m={m} d={d}")
    run_and_check(integer_valued(p, seed=33), d, 6, integer=True, planned=False, label=f"plan-free row runs int m={m} d={d}")
