"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by element.

Bar: bit-exact on small-integer inputs; |C - C_ref| <= 1e-5 * (|A|.|B|)_ij + 1e-7 on fp32 inputs.
"""
import numpy as np
import pytest
import torch

import paper_2405_16883_amd as sp
from oracle import hot_columns_oracle, plan_oracle
from workloads import (csr_from_row_lengths, integer_valued, make_scaled_config, with_padding)

from gpu_util import DeviceProblem, check_against_oracle, read_plan_arrays, tuning

pytestmark = pytest.mark.gpu

# (config, scale): sizes the oracle finishes in well under a second, still many tiles and a ragged tail
SMALL = [(1, 1.0), (2, 0.12), (3, 0.08), (4, 0.006), (5, 0.06)]
# parameter sets that force every execution path (windows, wave rows, single- and multi-piece block rows)
TUNES = [None, "bn=64,alpha=2,lw=8,ch=32,bch=64,u=4,nt=0", "bn=256,lw=64,ch=256,bch=256,u=8,nt=3",
         "bn=128,lw=0,ch=64,bch=128", "bn=32,alpha=1,lw=64,ch=64,bch=1000000", "hot=16,ch=64,bch=128", "hot=1",
         "bn=64,alpha=2,lw=8,ch=32,bch=64,fix=1"]  # fix=1: partial rows of split rows added inside the fused launch


def run_both(p, ldc=None, exact=False, label=""):
    d = DeviceProblem(p, ldc=ldc)
    plan = d.make_plan()
    worst = check_against_oracle(p, d.run_planned(plan), d.ldc, exact=exact, label=label + " planned")
    check_against_oracle(p, d.run_natural(), d.ldc, exact=exact, label=label + " plan-free")
    plan.destroy()
    return worst


@pytest.mark.parametrize("cfg,scale", SMALL)
def test_small_configs_fp32_tolerance(cfg, scale):
    p = make_scaled_config(cfg, scale, seed=0)
    print(f"cfg {cfg} x{scale}: m={p.m} k={p.k} n={p.n} nnz={p.nnz} maxrow={p.row_lengths.max()}", flush=True)
    run_both(p, label=p.name)


@pytest.mark.parametrize("cfg,scale", SMALL)
def test_small_configs_integer_bit_exact(cfg, scale):
    p = integer_valued(make_scaled_config(cfg, scale, seed=1), seed=1)
    run_both(p, exact=True, label=p.name)


@pytest.mark.parametrize("tune", TUNES)
@pytest.mark.parametrize("cfg,scale", [(3, 0.08), (4, 0.006), (1, 1.0)])
def test_every_path_under_forced_parameters(cfg, scale, tune):
    with tuning(tune):
        p = make_scaled_config(cfg, scale, seed=2)
        run_both(p, label=f"{p.name} [{tune}]")
        run_both(integer_valued(p, seed=2), exact=True, label=f"{p.name} int [{tune}]")


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 17, 63, 64, 65, 100, 128, 130, 255, 256, 257, 300, 512, 516, 1000])
def test_column_counts(n):
    rng = np.random.default_rng(n)
    lens = np.concatenate([rng.integers(0, 40, size=150), [700, 0, 300, 65, 64, 33, 32, 1]])
    p = csr_from_row_lengths(lens, 500, n, seed=n, duplicates=True)
    with tuning("ch=128,bch=256"):
        run_both(p, label=f"n={n}")
        run_both(integer_valued(p, seed=n), exact=True, label=f"n={n} int")


@pytest.mark.parametrize("n,ldb,ldc", [(64, 80, 72), (100, 101, 100), (100, 104, 108), (7, 9, 8), (128, 130, 131), (256, 260, 264)])
def test_leading_dimensions_and_padding(n, ldb, ldc):
    rng = np.random.default_rng(7)
    p = csr_from_row_lengths(rng.integers(0, 90, size=300), 400, n, seed=3)
    p = with_padding(p, ldb)  # B padding holds NaN: reading it into a result would show
    run_both(p, ldc=ldc, label=f"n={n} ldb={ldb} ldc={ldc}")
    run_both(integer_valued(p, seed=4), ldc=ldc, exact=True, label=f"n={n} ldb={ldb} ldc={ldc} int")


def test_base_pointers_at_float_alignment_only():
    p = csr_from_row_lengths(np.random.default_rng(1).integers(0, 50, size=200), 300, 64, seed=5)
    d = DeviceProblem(p)
    # shift B and C by one float: 4-byte aligned only
    Bbuf = torch.empty(p.k * p.n + 1, dtype=torch.float32, device=d.dev)
    Bv = Bbuf[1:].view(p.k, p.n)
    Bv.copy_(d.B)
    Cbuf = torch.full((p.m * p.n + 1,), -7.0, dtype=torch.float32, device=d.dev)
    Cv = Cbuf[1:].view(p.m, p.n)
    plan = d.make_plan()
    sp.scorch_spmm_csr_planned(plan, d.rowptr, d.colidx, d.vals, Bv, Cv)
    torch.cuda.synchronize()
    check_against_oracle(p, Cv.cpu().numpy(), p.n, label="unaligned planned")
    Cv.fill_(-7.0)
    sp.scorch_spmm_csr(p.m, p.k, p.n, d.rowptr, d.colidx, d.vals, Bv, Cv)
    torch.cuda.synchronize()
    check_against_oracle(p, Cv.cpu().numpy(), p.n, label="unaligned plan-free")
    assert float(Cbuf[0]) == -7.0
    plan.destroy()


@pytest.mark.parametrize("n", [64, 96, 128, 160, 256, 288, 544, 1024])
def test_xcd_sliced_column_mapping(n):
    """Forces the XCD-sliced grid (32-, 64- and 128-column slices dealt over the 8 XCDs) on shapes with 1..32 slices,
    the last one ragged where n is no multiple of the slice width."""
    rng = np.random.default_rng(n)
    lens = np.concatenate([rng.integers(0, 70, size=400), [900, 0, 300, 2100, 64, 33, 32, 1]])
    p = csr_from_row_lengths(lens, 700, n, seed=n + 1, duplicates=True)
    for tune in ("sliced=1,pack=0", "sliced=1,pack=1", "sliced=1,pack=1,ch=128,bch=256,lw=8", "sliced=64",
                 "sliced=64,ch=128,bch=256,lw=8", "sliced=128"):
        with tuning(tune):
            run_both(p, label=f"sliced n={n} [{tune}]")
            run_both(integer_valued(p, seed=n), exact=True, label=f"sliced n={n} int [{tune}]")
            run_both(with_padding(p, n + 4), ldc=n + 8, label=f"sliced n={n} padded [{tune}]")


@pytest.mark.parametrize("shape", [1, 2, 3])
@pytest.mark.parametrize("m,k,n", [(64, 64, 256), (130, 200, 128), (515, 1000, 512), (300, 77, 260), (257, 4100, 1028),
                                   (1000, 333, 2048)])
def test_panel_kernel_forced(m, k, n, shape):
    """The LDS panel kernel on shapes with ragged row blocks, ragged last panel and ragged last column tile."""
    rng = np.random.default_rng(m + n)
    lens = rng.integers(0, max(2, k // 3), size=m)
    lens[rng.integers(0, m, size=5)] = 0
    lens[0] = min(k, 700)  # a row whose 64-entry register window slides many times
    p = csr_from_row_lengths(lens, k, n, seed=m, duplicates=False)
    with tuning(f"panel={shape},pack=1"):  # panels fetched from a tile-major copy of B made at every call
        run_both(p, label=f"panel packed {m}x{k}x{n}")
        run_both(integer_valued(p, seed=n + 1), exact=True, label=f"panel packed int {m}x{k}x{n}")
        run_both(with_padding(p, n + 4), ldc=n + 12, label=f"panel packed padded {m}x{k}x{n}")
    with tuning(f"panel={shape}"):
        d = DeviceProblem(p)
        plan = d.make_plan()
        assert plan.info().mode == 2
        check_against_oracle(p, d.run_planned(plan), d.ldc, label=f"panel {m}x{k}x{n}")
        plan.destroy()
        q = integer_valued(p, seed=n)
        run_both(q, exact=True, label=f"panel int {m}x{k}x{n}")
        run_both(with_padding(p, n + 4), ldc=n + 12, label=f"panel padded {m}x{k}x{n}")
        # sorted rows that repeat a column are not for the panel kernel: the planner must hand them to the gather kernels
        r = csr_from_row_lengths(np.minimum(lens * 2, 3 * k), k, n, seed=m + 1, duplicates=True, sorted_cols=True)
        d = DeviceProblem(r)
        plan = d.make_plan()
        assert plan.info().mode != 2
        check_against_oracle(r, d.run_planned(plan), d.ldc, label=f"panel duplicates {m}x{k}x{n}")
        plan.destroy()


@pytest.mark.parametrize("shape", [1, 2, 3])
@pytest.mark.parametrize("k", [1, 31, 32, 33, 39, 40, 41, 64, 65, 80, 81, 200])
def test_panel_kernel_fully_dense_rows(k, shape):
    """Every row stores all k columns: each panel takes a whole 32- or 64-entry stretch of a row's register window,
    so the window is replaced at every panel; k around the panel heights covers the ragged last panel."""
    m, n = 70, 516
    lens = np.full(m, k)
    lens[[3, 69]] = 0
    p = csr_from_row_lengths(lens, k, n, seed=k, duplicates=False)
    with tuning(f"panel={shape}"):
        d = DeviceProblem(p)
        plan = d.make_plan()
        assert plan.info().mode == 2
        check_against_oracle(p, d.run_planned(plan), d.ldc, label=f"panel dense k={k}")
        plan.destroy()
        run_both(integer_valued(p, seed=k), exact=True, label=f"panel dense int k={k}")


def test_panel_mode_is_dropped_for_unsorted_rows_or_missing_colidx():
    p = csr_from_row_lengths([40] * 600, 300, 256, seed=3, sorted_cols=False)
    with tuning("panel=1"):
        d = DeviceProblem(p)
        plan = d.make_plan()
        assert plan.info().mode != 2  # unsorted: the planner falls back to the gather kernels
        check_against_oracle(p, d.run_planned(plan), d.ldc, label="unsorted fallback")
        plan.destroy()
        s = csr_from_row_lengths([40] * 600, 300, 256, seed=3, sorted_cols=True)
        d = DeviceProblem(s)
        plan = d.make_plan(with_colidx=False)
        assert plan.info().mode != 2  # cannot verify sortedness without colidx
        check_against_oracle(s, d.run_planned(plan), d.ldc, label="no-colidx fallback")
        plan.destroy()
        plan = d.make_plan()
        assert plan.info().mode == 2
        plan.destroy()


EDGE_LENS = {
    "m1": [5], "m1_empty": [0], "all_empty": [0] * 777, "last_empty": [3, 9, 0], "first_heavy": [5000, 1, 2, 0, 3],
    "only_heavy": [20000], "many_empty_then_row": [0] * 300 + [400] + [0] * 300, "len_boundaries": [31, 32, 33, 63, 64, 65, 127, 128, 129, 511, 512, 513, 2047, 2048, 2049],
    "alternating": [0, 1] * 200,
}


@pytest.mark.parametrize("name", sorted(EDGE_LENS))
def test_edge_shapes(name):
    lens = EDGE_LENS[name]
    for n, k in ((128, 3000), (100, 1), (4, 37)):
        p = csr_from_row_lengths(lens, k, n, seed=11, duplicates=True, sorted_cols=False)
        run_both(p, label=f"{name} n={n} k={k}")
        run_both(integer_valued(p, seed=12), exact=True, label=f"{name} n={n} k={k} int")


@pytest.mark.parametrize("m,n", [(16384 + 37, 1), (16384 + 37, 33), (16384 + 37, 128), (16384 + 37, 300),
                                 (65536 + 5, 1), (65536 + 5, 8), (65536 + 5, 24)])
def test_plan_free_row_runs(m, n):
    """With 16 384 rows or more the plan-free kernel gives a wavefront a run of 4 consecutive rows (up to 16 with 65 536
    rows or more and narrow lane groups, i.e. small n): short rows are staged
    together (at most 320 entries, rows of up to 32), longer ones streamed, rows beyond 256 / 2 048 entries left to
    the whole workgroup depending on how many of them the workgroup has.  Row lengths sit on every one of these limits,
    in runs that mix them, in a matrix whose last workgroup is ragged."""
    rng = np.random.default_rng(21)
    lens = rng.integers(0, 41, size=m)
    special = [0, 1, 31, 32, 33, 64, 255, 256, 257, 287, 288, 289, 319, 320, 321, 2047, 2048, 2049, 3000]
    for i, pos in enumerate(range(5, m - 64, 211)):
        lens[pos] = special[i % len(special)]
    lens[1000:1016] = 20  # a run of 16 rows = 4 wavefronts x 4 rows whose stages are exactly full (80 entries each)
    lens[2000:2004] = [80, 80, 80, 80]  # 320 entries: the largest stage
    lens[3000:3016] = 300  # a workgroup with many rows beyond 256 entries: every wavefront keeps its own
    lens[4000:4016] = [0] * 15 + [257]  # a single such row in a workgroup: taken by the 4 wavefronts together
    lens[m - 3:] = [2049, 0, 33]
    p = csr_from_row_lengths(lens.tolist(), 5000, n, seed=22, duplicates=True, sorted_cols=False)
    d = DeviceProblem(p)
    check_against_oracle(p, d.run_natural(), d.ldc, label=f"plan-free row runs n={n}")
    q = integer_valued(p, seed=23)
    dq = DeviceProblem(q)
    check_against_oracle(q, dq.run_natural(), dq.ldc, exact=True, label=f"plan-free row runs n={n} int")


def test_single_row_with_very_many_entries():
    # integer case: |partial sums| <= 4*8*500000 = 1.6e7 < 2^24, so every summation order is exact
    p = integer_valued(csr_from_row_lengths([500_000, 2, 0], 50_000, 128, seed=13, duplicates=True), seed=13)
    run_both(p, exact=True, label="5e5-entry row int")
    q = csr_from_row_lengths([1_000_000, 2, 0], 50_000, 128, seed=14, duplicates=True)
    run_both(q, label="1e6-entry row fp32")


def test_zero_sizes_and_argument_errors():
    dev = torch.device("cuda:0")
    z32 = torch.zeros(1, dtype=torch.int32, device=dev)
    f = torch.zeros((4, 4), dtype=torch.float32, device=dev)
    sp.scorch_spmm_csr(0, 4, 4, z32, z32, f.view(-1), f, f)  # m = 0: no work
    sp.scorch_spmm_csr(4, 4, 0, torch.zeros(5, dtype=torch.int32, device=dev), z32, f.view(-1), f[:, :0], f[:, :0])
    plan = sp.scorch_spmm_plan(0, 4, 4, z32, 0)
    sp.scorch_spmm_csr_planned(plan, z32, z32, f.view(-1), f, f)
    plan.destroy()
    lib = sp.load_library()
    rp = torch.zeros(5, dtype=torch.int32, device=dev)
    # ldb < n and ldc < n are rejected before anything is enqueued
    st = lib.scorch_spmm_csr(4, 4, 4, rp.data_ptr(), z32.data_ptr(), f.data_ptr(), f.data_ptr(), 3, f.data_ptr(), 4, None)
    assert st == sp.binding.SCORCH_ERR_INVALID_ARG
    st = lib.scorch_spmm_csr(4, 4, 4, rp.data_ptr(), z32.data_ptr(), f.data_ptr(), f.data_ptr(), 4, f.data_ptr(), 2, None)
    assert st == sp.binding.SCORCH_ERR_INVALID_ARG
    st = lib.scorch_spmm_csr(-1, 4, 4, rp.data_ptr(), z32.data_ptr(), f.data_ptr(), f.data_ptr(), 4, f.data_ptr(), 4, None)
    assert st == sp.binding.SCORCH_ERR_INVALID_ARG
    st = lib.scorch_spmm_csr(4, 4, 4, None, z32.data_ptr(), f.data_ptr(), f.data_ptr(), 4, f.data_ptr(), 4, None)
    assert st == sp.binding.SCORCH_ERR_INVALID_ARG and b"NULL" in lib.scorch_last_error()
    # workspace too small / misaligned
    ws = torch.empty(512, dtype=torch.uint8, device=dev)
    with pytest.raises(sp.ScorchError) as e:
        sp.scorch_spmm_plan(100000, 4, 4, torch.zeros(100001, dtype=torch.int32, device=dev), 0, workspace=ws)
    assert e.value.status == sp.binding.SCORCH_ERR_WORKSPACE_TOO_SMALL
    with pytest.raises(sp.ScorchError) as e:
        sp.scorch_spmm_plan(4, 4, 4, rp, 0, workspace=torch.empty(4096, dtype=torch.uint8, device=dev)[1:])
    assert e.value.status == sp.binding.SCORCH_ERR_INVALID_ARG


@pytest.mark.parametrize("tune", TUNES)
@pytest.mark.parametrize("cfg,scale", [(3, 0.08), (4, 0.006), (2, 0.12)])
def test_plan_lists_match_the_plan_oracle_bit_for_bit(cfg, scale, tune):
    with tuning(tune):
        p = make_scaled_config(cfg, scale, seed=3)
        d = DeviceProblem(p)
        plan = d.make_plan()
        info, got = read_plan_arrays(plan)
        want = plan_oracle(p.rowptr, info.BN, info.ALPHA, info.LW, info.CH, info.BCH)
        assert info.nnz == p.nnz and info.n_short_rows == int(want["n_short"])
        assert info.n_partial_slots == int(want["n_slots"])
        for key in ("win_row_start", "win_stage", "wave_rows", "wave_span", "items", "split"):
            assert got[key].shape == want[key].shape, key
            assert np.array_equal(got[key], want[key]), key
        plan.destroy()


def test_plan_edge_patterns_match_oracle():
    for lens in ([0] * 1000, [100000], [0, 0, 5000, 0], [33] * 600, []):
        p = csr_from_row_lengths(lens, 4000, 8, seed=1, duplicates=True)
        with tuning("bn=64,alpha=2,lw=16,ch=64,bch=128"):
            d = DeviceProblem(p)
            plan = d.make_plan()
            info, got = read_plan_arrays(plan)
            want = plan_oracle(p.rowptr, info.BN, info.ALPHA, info.LW, info.CH, info.BCH)
            for key in ("win_row_start", "win_stage", "wave_rows", "wave_span", "items", "split"):
                assert np.array_equal(got[key], want[key]), (key, lens[:4])
            plan.destroy()


def test_repeated_runs_are_bit_identical():
    p = make_scaled_config(3, 0.08, seed=5)
    d = DeviceProblem(p)
    plan = d.make_plan()
    first = d.run_planned(plan).copy()
    for _ in range(3):
        assert np.array_equal(first, d.run_planned(plan))
    plan.destroy()


@pytest.mark.parametrize("budget_kb", [1, 8, 64, 100000])
def test_hot_column_marking_changes_cache_policy_only(budget_kb):
    """Forced hot/cold split: the set of hot columns follows the stated rule (whole degree bins from the top while they
    fit the byte budget, 16 bins per power of two), and the result is bit-identical to the run without the split."""
    p = make_scaled_config(3, 0.08, seed=12)  # power-law columns
    d = DeviceProblem(p)
    plan0 = d.make_plan()
    base = d.run_planned(plan0).copy()
    assert plan0.info().n_hot_columns == 0  # B is far smaller than the memory-side cache: no split by default
    plan0.destroy()
    with tuning(f"hot={budget_kb}"):
        plan = d.make_plan()
        info = plan.info()
        rows, share = hot_columns_oracle(p.colidx, p.k, p.n, budget_kb)
        assert info.n_hot_columns == rows
        assert abs(info.hot_share - share) < 1e-6
        out = d.run_planned(plan)
        assert np.array_equal(out, base)
        check_against_oracle(p, out, d.ldc, label=f"hot={budget_kb}")
        plan.destroy()
    # the cold rows read with the other cache-policy bits (experiments; buffer loads): the same bits again
    for cold in (1, 2, 3):
        with tuning(f"hot={budget_kb},cold={cold}"):
            plan = d.make_plan()
            assert np.array_equal(d.run_planned(plan), base), f"cold={cold} changed the result"
            plan.destroy()


def test_runs_on_a_side_stream():
    p = make_scaled_config(1, 1.0, seed=6)
    d = DeviceProblem(p)
    s = torch.cuda.Stream()
    plan = sp.scorch_spmm_plan(p.m, p.k, p.n, d.rowptr, p.nnz, stream=s)
    d.reset_C()
    torch.cuda.synchronize()
    sp.scorch_spmm_csr_planned(plan, d.rowptr, d.colidx, d.vals, d._B_arg(), d._C_arg(), stream=s)
    s.synchronize()
    check_against_oracle(p, d.Cfull.cpu().numpy(), d.ldc, label="side stream")
    plan.destroy()


@pytest.mark.parametrize("k,density", [(784, 0.2), (3072, 0.1), (3072, 0.5), (12288, 0.05)])
def test_sparse_activation_times_dense_weight_shape(k, density):
    """The sparse linear layer of the paper's autoencoder (Section 5.2, Table 2): a batch of 64 sparse input rows
    times a dense k x 256 weight.  Few, long rows: the planner cuts them into pieces or hands them to the panel kernel."""
    rng = np.random.default_rng(k)
    lens = rng.binomial(k, density, size=64)
    p = csr_from_row_lengths(lens, k, 256, seed=k)
    run_both(p, label=f"batch 64 x {k} @ {k} x 256, density {density}")
    run_both(integer_valued(p, seed=1), exact=True, label=f"batch 64 x {k} int")


@pytest.mark.parametrize("n,tune", [(128, "ch=64,bch=64"), (100, "ch=64,bch=128"), (1040, "ch=64,bch=64"), (256, "sliced=1,pack=1,ch=64,bch=64"),
                                    (256, "sliced=64,ch=64,bch=96"), (3, "ch=64,bch=64"), (64, "hot=4,ch=64,bch=64")])
def test_split_rows_added_inside_the_launch_match_the_second_launch_bit_for_bit(n, tune):
    """Rows cut into many pieces (up to 150 per row, several column tiles or XCD slices).  Default: a second launch
    adds the partial rows.  fix=1: the piece that arrives last adds them, in piece order, so the result equals
    that of the second launch bit for bit at every repetition (the arrival order changes from run to run, the sum
    must not), and the arrival counters are back at zero after every launch (else the next one would go wrong)."""
    rng = np.random.default_rng(n)
    lens = np.concatenate([rng.integers(0, 60, size=300), [9600, 5000, 0, 1300, 700, 130, 129, 128, 65, 64]])
    rng.shuffle(lens)
    p = csr_from_row_lengths(lens, 900, n, seed=n + 7, duplicates=True)
    d = DeviceProblem(p)
    with tuning(tune):
        plan = d.make_plan()
        assert plan.info().n_split_rows >= 5
        want = d.run_planned(plan).copy()
        plan.destroy()
    check_against_oracle(p, want, d.ldc, label=f"two launches n={n} [{tune}]")
    for fix in (1,):
        with tuning(tune + f",fix={fix}"):
            plan = d.make_plan()
            for rep in range(12):
                got = d.run_planned(plan)
                assert np.array_equal(got, want), f"fix={fix} differs from the fix-up launch at repetition {rep} (n={n}, {tune})"
            plan.destroy()
            run_both(integer_valued(p, seed=n), exact=True, label=f"fix={fix} int n={n} [{tune}]")


@pytest.mark.parametrize("k,n", [(16384, 128), (8192, 256), (2048, 1024), (1024, 2176), (4100, 640), (33000, 64), (16384, 192)])
def test_plan_free_call_with_column_slices_over_the_dies(k, n):
    """Shapes whose B reaches 8 MB: the plan-free call deals 64- or 128-column slices over the XCDs (2 to 17 slices,
    i.e. whole rounds of 8 plus shared rounds); shapes just outside the rule (n = 64, n not a multiple) keep whole rows."""
    rng = np.random.default_rng(n + k)
    lens = np.concatenate([rng.integers(0, 70, size=300), [2500, 0, 300, 700, 64, 33, 32, 1, 0]])
    p = csr_from_row_lengths(lens, k, n, seed=n, duplicates=True)
    d = DeviceProblem(p)
    check_against_oracle(p, d.run_natural(), d.ldc, label=f"plan-free sliced k={k} n={n}")
    q = integer_valued(p, seed=k)
    d = DeviceProblem(q, ldc=n + 4)
    check_against_oracle(q, d.run_natural(), d.ldc, exact=True, label=f"plan-free sliced int k={k} n={n}")
