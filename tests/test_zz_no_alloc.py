"""scorch_spmm_csr_static, the entry point for callers that cannot allocate device memory, against
scorch_spmm_plan + scorch_spmm_csr_planned (the existing entry point whose workspace it replaces with the library's
static scratch array), through the C ABI: two calls in a row, the second with a smaller input, each compared with the
planned call bit for bit (same kernels, same plan) and with the fp64 oracle to the parity tolerance; torch's allocator
must not see a single allocation during the calls; a problem whose plan does not fit the array is refused."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2405_16883_amd as sp
from workloads import csr_from_row_lengths, integer_valued, make_scaled_config

from gpu_util import SENTINEL, DeviceProblem, check_against_oracle

pytestmark = pytest.mark.gpu


def static_call(d):
    """Raw C-ABI call (ctypes, plain pointers and sizes) of the allocation-free entry point on a DeviceProblem."""
    lib = sp.load_library()
    p = d.p
    d.reset_C()
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    st = lib.scorch_spmm_csr_static(p.m, p.k, p.n, d.rowptr.data_ptr(), d.colidx.data_ptr() if p.nnz else None,
                                    d.vals.data_ptr() if p.nnz else None, d.Bfull.data_ptr(), p.ldb,
                                    d.Cfull.data_ptr(), d.ldc, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == 0, lib.scorch_last_error().decode()
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before, "the call went through torch's allocator"
    return d.Cfull.cpu().numpy()


def compare(p, label, ldc=None, exact=False):
    d = DeviceProblem(p, ldc=ldc)
    plan = d.make_plan()
    info = plan.info()
    assert info.workspace_bytes_used <= sp.STATIC_SCRATCH_BYTES
    want = d.run_planned(plan).copy()
    plan.destroy()
    got = static_call(d)
    assert np.array_equal(got, want), f"{label}: static-scratch result differs from the planned call"
    check_against_oracle(p, got, d.ldc, exact=exact, label=label)
    return info


def test_two_calls_in_a_row_the_second_smaller():
    # first: a power-law pattern with rows long enough to be cut into pieces (partial rows in the scratch array)
    rng = np.random.default_rng(5)
    lens = np.concatenate([rng.integers(0, 40, size=6000), [9000, 5000, 0, 0, 2500, 300, 64, 33]])
    rng.shuffle(lens)
    big = csr_from_row_lengths(lens, 7000, 128, seed=5)
    info = compare(big, "first call (split rows)", ldc=136)
    assert info.n_split_rows > 0 and info.n_partial_slots > 0 and info.n_windows > 1 and info.n_wave_rows > 0
    # second: a smaller input straight after it, whose lists and partial rows overwrite only the front of what the
    # first call left behind
    small = make_scaled_config(3, 0.02, seed=9)
    assert small.m < big.m and small.nnz < big.nnz
    compare(small, "second call (smaller)")
    # and the first one again, integer-valued: bit-exact against the oracle as well
    compare(integer_valued(big, seed=6), "third call (integers)", exact=True)


def test_shapes_that_use_other_parts_of_the_scratch():
    # XCD-sliced gather with the repacked copy of B, and the LDS panel kernel: both keep a copy of B in the workspace
    compare(make_scaled_config(2, 0.25, seed=1), "uniform pattern, sliced")
    compare(make_scaled_config(5, 0.25, seed=1), "pruned weight")
    # n <= 4 (one-lane groups), empty matrix, single row
    compare(csr_from_row_lengths([5, 0, 700, 3, 64, 0, 1], 300, 1, seed=2), "n = 1")
    compare(csr_from_row_lengths([0, 0, 0], 10, 8, seed=3), "all rows empty")
    compare(csr_from_row_lengths([100000], 500, 100, seed=4), "one long row")


def test_oversized_problem_is_refused_and_nothing_is_written():
    lib = sp.load_library()
    # wide B with long rows: the XCD-sliced gather wants a 32 MB slice-major copy of B in the workspace
    p = csr_from_row_lengths([64] * 64, 16384, 512, seed=8)
    assert sp.scorch_spmm_plan_workspace_bytes(p.m, p.k, p.n, p.nnz) > sp.STATIC_SCRATCH_BYTES
    d = DeviceProblem(p)
    rowptr, B, C = d.rowptr, d.Bfull, d.Cfull
    st = lib.scorch_spmm_csr_static(p.m, p.k, p.n, rowptr.data_ptr(), d.colidx.data_ptr(), d.vals.data_ptr(), B.data_ptr(),
                                    p.ldb, C.data_ptr(), d.ldc, None)
    torch.cuda.synchronize()
    assert st == sp.binding.SCORCH_ERR_UNSUPPORTED
    msg = lib.scorch_last_error().decode()
    assert str(sp.STATIC_SCRATCH_BYTES) in msg and "scorch_spmm_plan" in msg
    assert bool((C == SENTINEL).all())
    # bad arguments are refused before anything is touched
    assert lib.scorch_spmm_csr_static(4, 4, 4, None, None, None, None, 4, None, 4, None) == sp.binding.SCORCH_ERR_INVALID_ARG
    assert lib.scorch_spmm_csr_static(4, 4, 8, rowptr.data_ptr(), None, None, B.data_ptr(), 4, C.data_ptr(), 8, None) == sp.binding.SCORCH_ERR_INVALID_ARG
    assert lib.scorch_spmm_csr_static(0, 4, 4, None, None, None, None, 4, None, 4, None) == 0
