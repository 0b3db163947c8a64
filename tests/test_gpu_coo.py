"""Coordinate-list input: row pointers built on the device match the oracle bit for bit, and SpMM through them
matches the SpMM oracle."""
import numpy as np
import pytest
import torch

import paper_2405_16883_amd as sp
from oracle import coo_rowptr_oracle, dcsr_rowptr_oracle
from workloads import csr_from_row_lengths, make_scaled_config

from gpu_util import DeviceProblem, check_against_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def device_rowptr(m, rows):
    r = torch.from_numpy(np.ascontiguousarray(rows, dtype=np.int32)).to(DEV)
    out = torch.full((m + 1,), -5, dtype=torch.int32, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    sp.scorch_coo_to_csr_rowptr(m, r, out, flag)
    torch.cuda.synchronize()
    return out.cpu().numpy(), int(flag.item())


@pytest.mark.parametrize("lens", [[0] * 50, [7], [0, 0, 5, 0, 0, 0, 9, 0], [3] * 1000, [0] * 999 + [1], [100000, 0, 1]])
def test_rowptr_edge_patterns(lens):
    p = csr_from_row_lengths(lens, 1000, 4, seed=1, duplicates=True)
    rows = np.repeat(np.arange(p.m), p.row_lengths)
    got, bad = device_rowptr(p.m, rows)
    assert bad == 0 and np.array_equal(got, coo_rowptr_oracle(p.m, rows)) and np.array_equal(got, p.rowptr)


def test_unsorted_or_out_of_range_rows_raise_the_flag():
    assert device_rowptr(4, [0, 2, 1, 3])[1] == 1
    assert device_rowptr(4, [0, 1, 4])[1] == 1
    assert device_rowptr(4, [-1, 1])[1] == 1
    assert device_rowptr(4, [0, 1, 1, 3])[1] == 0


@pytest.mark.parametrize("rows", [[-5, 3], [-5, -5, 3], [0, -2, 3], [9, 9], [2, 1000000], [-2147483648, 0],
                                  [2147483647, 2147483647], [3, -7]])
def test_bad_row_ids_raise_the_flag_and_write_nothing_outside_rowptr(rows):
    """A key outside [0, m) must not steer the fill outside rowptr_out[0..m], whether it is the entry that closes a
    range or its predecessor: rowptr_out sits in the middle of a guarded buffer."""
    m, guard = 4, 4096
    buf = torch.full((guard + m + 1 + guard,), -77, dtype=torch.int32, device=DEV)
    out = buf[guard:guard + m + 1]
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    sp.scorch_coo_to_csr_rowptr(m, torch.tensor(rows, dtype=torch.int32, device=DEV), out, flag)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert int(flag.item()) == 1
    assert np.all(host[:guard] == -77) and np.all(host[guard + m + 1:] == -77)
    # the same through the doubly compressed entry point (strictly increasing ids)
    buf.fill_(-77)
    flag.zero_()
    ids = torch.tensor(rows, dtype=torch.int32, device=DEV)
    pos = torch.arange(len(rows) + 1, dtype=torch.int32, device=DEV)
    sp.scorch_dcsr_to_csr_rowptr(m, ids, pos, out, flag)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert int(flag.item()) == 1
    assert np.all(host[:guard] == -77) and np.all(host[guard + m + 1:] == -77)


@pytest.mark.parametrize("cfg,scale", [(1, 1.0), (3, 0.08), (5, 0.06)])
def test_spmm_from_a_coordinate_list(cfg, scale):
    p = make_scaled_config(cfg, scale, seed=5)
    rows = np.repeat(np.arange(p.m), p.row_lengths)
    d = DeviceProblem(p)
    r = torch.from_numpy(rows.astype(np.int32)).to(DEV)
    rowptr = torch.empty(p.m + 1, dtype=torch.int32, device=DEV)
    sp.scorch_coo_to_csr_rowptr(p.m, r, rowptr)
    plan = sp.scorch_spmm_plan(p.m, p.k, p.n, rowptr, p.nnz, colidx=d.colidx)
    d.reset_C()
    sp.scorch_spmm_csr_planned(plan, rowptr, d.colidx, d.vals, d._B_arg(), d._C_arg())
    torch.cuda.synchronize()
    check_against_oracle(p, d.Cfull.cpu().numpy(), d.ldc, label=f"{p.name} from COO")
    plan.destroy()


@pytest.mark.parametrize("lens", [[0] * 50, [7], [0, 0, 5, 0, 0, 0, 9, 0], [3] * 1000, [0] * 999 + [1], [4, 0, 0, 1]])
def test_dcsr_rowptr(lens):
    L = np.asarray(lens)
    m = len(L)
    ids = np.nonzero(L)[0].astype(np.int32)
    pos = np.concatenate([[0], np.cumsum(L[ids])]).astype(np.int32)
    out = torch.full((m + 1,), -5, dtype=torch.int32, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    sp.scorch_dcsr_to_csr_rowptr(m, torch.from_numpy(ids).to(DEV), torch.from_numpy(pos).to(DEV), out, flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0
    assert np.array_equal(out.cpu().numpy(), dcsr_rowptr_oracle(m, ids, pos))


def test_dcsr_flags_repeated_or_unsorted_rows():
    for ids in ([1, 1], [2, 1], [0, 7]):
        out = torch.zeros(5, dtype=torch.int32, device=DEV)
        flag = torch.zeros(1, dtype=torch.int32, device=DEV)
        sp.scorch_dcsr_to_csr_rowptr(4, torch.tensor(ids, dtype=torch.int32, device=DEV),
                                     torch.tensor([0, 1, 2], dtype=torch.int32, device=DEV), out, flag)
        torch.cuda.synchronize()
        assert int(flag.item()) == 1
