"""Randomised GPU parity: many small problems with random shapes, row-length mixes, paddings and forced plan
parameters, each compared element by element with the fp64 oracle (fp32 tolerance) and, on its integer-valued twin,
bit for bit.  Seeded: every case is reproducible from its index."""
import numpy as np
import pytest

from workloads import csr_from_row_lengths, integer_valued, with_padding

from gpu_util import DeviceProblem, check_against_oracle, tuning

pytestmark = pytest.mark.gpu

TUNES = [None, None, "bn=16,lw=4,ch=16,bch=32", "bn=256,lw=64,ch=64,bch=64", "lw=0,ch=32,bch=48,u=4", "sliced=1,pack=1",
         "sliced=1,pack=0,ch=64,bch=128", "panel=1", "panel=2", "hot=1", "hot=4,bn=32,ch=32,bch=64", "nt=0,alpha=1,bn=64"]


def draw_case(i):
    rng = np.random.default_rng(1000 + i)
    m = int(rng.choice([1, 2, 3, 5, 17, 63, 64, 65, 130, 257, 400]))
    k = int(rng.choice([1, 2, 7, 31, 32, 33, 64, 100, 500, 1500, 3000]))
    n = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 31, 32, 33, 64, 65, 100, 127, 128, 129, 256, 260, 511, 512, 516, 700]))
    kind = int(rng.integers(0, 5))
    if kind == 0:
        lens = rng.integers(0, min(k, 40) + 1, size=m)
    elif kind == 1:
        lens = np.minimum((rng.pareto(1.2, size=m) * 3).astype(np.int64), 4 * k)  # heavy tail, rows longer than k
    elif kind == 2:
        lens = np.full(m, min(k, int(rng.integers(1, 200))))
    elif kind == 3:
        lens = np.zeros(m, dtype=np.int64)
        lens[rng.integers(0, m, size=max(1, m // 8))] = int(rng.integers(1, 3000))
    else:
        lens = rng.integers(0, 3, size=m)
    duplicates = bool(rng.integers(0, 2)) or int(lens.max(initial=0)) > k
    sorted_cols = bool(rng.integers(0, 2))
    p = csr_from_row_lengths(lens, k, n, seed=i, duplicates=duplicates, sorted_cols=sorted_cols)
    pad_b = int(rng.choice([0, 0, 1, 3, 4]))
    pad_c = int(rng.choice([0, 0, 1, 4, 7]))
    tune = TUNES[int(rng.integers(0, len(TUNES)))]
    return p, pad_b, pad_c, tune


@pytest.mark.parametrize("block", range(16))
def test_random_small_problems(block):
    for i in range(block * 20, block * 20 + 20):
        p, pad_b, pad_c, tune = draw_case(i)
        label = f"case {i}: m={p.m} k={p.k} n={p.n} nnz={p.nnz} ldb+{pad_b} ldc+{pad_c} [{tune}]"
        print(label, flush=True)
        if pad_b:
            p = with_padding(p, p.n + pad_b)  # padding of B holds NaN
        with tuning(tune):
            for q, exact in ((p, False), (integer_valued(p, seed=i), True)):
                d = DeviceProblem(q, ldc=q.n + pad_c)
                plan = d.make_plan()
                check_against_oracle(q, d.run_planned(plan), d.ldc, exact=exact, label=label + " planned")
                check_against_oracle(q, d.run_natural(), d.ldc, exact=exact, label=label + " plan-free")
                plan.destroy()


def draw_tall_case(i):
    """Matrices tall enough that the plan-free kernels give a wavefront a run of several rows, and wide enough
    that the planner's column slicing applies to some of them."""
    rng = np.random.default_rng(5000 + i)
    m = int(rng.choice([8192, 12000, 16385, 40000, 70001]))
    k = int(rng.choice([64, 1000, 20000]))
    n = int(rng.choice([1, 4, 8, 24, 64, 100, 128, 192, 256]))
    kind = int(rng.integers(0, 3))
    if kind == 0:
        lens = rng.integers(0, 40, size=m)
    elif kind == 1:
        lens = np.minimum((rng.pareto(1.1, size=m) * 4).astype(np.int64), 6000)  # heavy tail: outlier rows
    else:
        lens = rng.choice([0, 1, 30, 33, 250, 260, 300], size=m, p=[0.3, 0.3, 0.2, 0.1, 0.04, 0.03, 0.03])
    p = csr_from_row_lengths(lens, k, n, seed=i, duplicates=True, sorted_cols=bool(rng.integers(0, 2)))
    return p


@pytest.mark.parametrize("i", range(8))
def test_random_tall_problems(i):
    p = draw_tall_case(i)
    label = f"tall case {i}: m={p.m} k={p.k} n={p.n} nnz={p.nnz}"
    print(label, flush=True)
    for q, exact in ((p, False), (integer_valued(p, seed=i), True)):
        d = DeviceProblem(q)
        plan = d.make_plan()
        check_against_oracle(q, d.run_planned(plan), d.ldc, exact=exact, label=label + " planned")
        check_against_oracle(q, d.run_natural(), d.ldc, exact=exact, label=label + " plan-free")
        plan.destroy()
