"""Structural invariants that pin the planner's definition (oracle/plan.py)."""
import numpy as np
import pytest

from oracle import plan_oracle
from workloads import csr_from_row_lengths, make_scaled_config


def check_plan(rowptr, P, BN, ALPHA, LW, CH, BCH):
    rp = np.asarray(rowptr, dtype=np.int64)
    m = rp.shape[0] - 1
    lens = np.diff(rp)
    w = P["win_row_start"].astype(np.int64)
    # windows partition the rows, in order
    assert w[0] == 0 and w[-1] == m and np.all(np.diff(w) >= 0)
    assert np.all(np.diff(w) <= -(-BN // ALPHA))  # rows per window bounded
    for i in range(len(w) - 1):
        if w[i + 1] > w[i]:
            span = rp[w[i + 1] - 1] - rp[w[i]]  # distance between first and last row start
            assert span < BN
    # what a window stages: exactly the span from its first to its last short row, which holds every entry of every
    # short row of the window (BN + LW <= 320 entries, so the cap never cuts a short row)
    st = P["win_stage"].astype(np.int64)
    assert st.shape == (len(w) - 1, 2) and BN + LW <= 320
    for i in range(len(w) - 1):
        rows = np.arange(w[i], w[i + 1])
        sh = rows[lens[rows] <= LW]
        if len(sh) == 0:
            assert st[i].tolist() == [0, -1]
        else:
            beg, cnt = st[i]
            assert beg == rp[sh[0]] and 0 <= cnt <= 320
            assert np.all(rp[sh] >= beg) and np.all(rp[sh + 1] <= beg + cnt)
            assert cnt == min(rp[sh[-1] + 1] - beg, 320)
    covered = np.zeros(m, dtype=np.int64)
    short = lens <= LW
    covered[short] += 1  # every short row is inside exactly one window (partition above)
    np.add.at(covered, P["wave_rows"], 1)
    assert np.all((lens[P["wave_rows"]] > LW) & (lens[P["wave_rows"]] <= CH))
    assert np.all(np.diff(P["wave_rows"]) > 0)
    assert np.array_equal(P["wave_span"], np.stack([rp[P["wave_rows"]], rp[P["wave_rows"] + 1]], axis=1))
    items = P["items"].astype(np.int64)
    seen_slots = []
    for row in np.unique(items[:, 0]) if len(items) else []:
        it = items[items[:, 0] == row]
        assert lens[row] > CH
        assert it[0, 1] == rp[row] and it[-1, 2] == rp[row + 1]
        assert np.all(it[1:, 1] == it[:-1, 2])  # pieces tile the row
        assert np.all(it[:, 2] - it[:, 1] <= BCH) and np.all(it[:, 2] > it[:, 1])
        if len(it) == 1:
            assert it[0, 3] == -1
        else:
            assert np.all(np.diff(it[:, 3]) == 1)
            seen_slots.extend(it[:, 3].tolist())
            s = P["split"][P["split"][:, 0] == row]
            assert len(s) == 1 and s[0, 1] == it[0, 3] and s[0, 2] == len(it)
        covered[row] += 1
    assert np.all(covered == 1)
    assert sorted(seen_slots) == list(range(int(P["n_slots"])))
    assert len(P["split"]) == len({r for r in items[:, 0] if (items[:, 0] == r).sum() > 1}) if len(items) else len(P["split"]) == 0


@pytest.mark.parametrize("params", [(128, 4, 32, 128, 512), (64, 2, 16, 64, 64), (256, 8, 64, 1024, 4096)])
@pytest.mark.parametrize("cfg,scale", [(1, 0.2), (3, 0.03), (4, 0.002)])
def test_plan_invariants_on_workloads(cfg, scale, params):
    p = make_scaled_config(cfg, scale, seed=0)
    BN, ALPHA, LW, CH, BCH = params
    check_plan(p.rowptr, plan_oracle(p.rowptr, *params), *params)


def test_plan_edge_cases():
    params = (64, 2, 16, 64, 128)
    for lens in ([0] * 500, [1000], [0, 0, 1000, 0], [17] * 100, [64, 65, 128, 129, 16, 17, 0], []):
        p = csr_from_row_lengths(lens, 2000, 4, seed=1, duplicates=True)
        check_plan(p.rowptr, plan_oracle(p.rowptr, *params), *params)
    P = plan_oracle(csr_from_row_lengths([64, 65, 128, 129, 16, 17, 0], 2000, 4, duplicates=True).rowptr, *params)
    assert P["row_class"].tolist() == [1, 2, 2, 2, 0, 1, 0]
    assert P["items"][:, 3].tolist() == [-1, -1, 0, 1]
    assert P["split"].tolist() == [[3, 0, 2, 0]]
    # row pointers 0 64 129 257 386 402 419 419, keys rowptr[i] + 2 i = 0 66 133 263 394 412 431, windows of 64 key units:
    # rows 0..3 sit alone in windows 0, 1, 2, 4; rows 4, 5, 6 share window 6, whose short rows are 4 (16 entries) and 6
    # (empty), so it stages entries 386 .. 419 (the medium row 5 lies in between and is staged along)
    assert P["win_row_start"].tolist() == [0, 1, 2, 3, 3, 4, 4, 7]
    assert P["win_stage"].tolist() == [[0, -1], [0, -1], [0, -1], [0, -1], [0, -1], [0, -1], [386, 33]]


def test_coo_rowptr_oracle_against_the_generators_own_row_pointers():
    from oracle import coo_rowptr_oracle
    for cfg, scale in ((1, 0.3), (3, 0.02), (5, 0.03)):
        p = make_scaled_config(cfg, scale, seed=2)
        rows = np.repeat(np.arange(p.m), p.row_lengths).astype(np.int32)  # the coordinate list of the same matrix
        assert np.array_equal(coo_rowptr_oracle(p.m, rows), p.rowptr)
    assert coo_rowptr_oracle(4, np.zeros(0, np.int32)).tolist() == [0, 0, 0, 0, 0]
    assert coo_rowptr_oracle(5, np.array([1, 1, 3], np.int32)).tolist() == [0, 0, 2, 2, 3, 3]


def test_dcsr_rowptr_oracle_round_trip():
    from oracle import dcsr_rowptr_oracle
    for cfg, scale in ((3, 0.02), (4, 0.002)):
        p = make_scaled_config(cfg, scale, seed=3)
        L = p.row_lengths
        ids = np.nonzero(L)[0]
        pos = np.concatenate([[0], np.cumsum(L[ids])])
        assert np.array_equal(dcsr_rowptr_oracle(p.m, ids, pos), p.rowptr)
    assert dcsr_rowptr_oracle(5, np.array([1, 3]), np.array([0, 2, 3])).tolist() == [0, 0, 2, 2, 3, 3]
    assert dcsr_rowptr_oracle(3, np.zeros(0, np.int64), np.array([0])).tolist() == [0, 0, 0, 0]


def test_hot_columns_rule_on_a_hand_worked_case():
    """Column counts 5, 3, 3, 1, 0 (12 entries).  Rows of B of 512 bytes and a 1 KB budget hold two rows: the bin of the
    count 5 (one column) is taken, the bin of the count 3 (two columns) would make three rows and is not; with 256-byte
    rows the budget holds four rows and the bins of 5, 3 and 1 are all taken; whole bins only, so two columns that tie
    are marked together or not at all."""
    from oracle import hot_columns_oracle
    colidx = np.array([0] * 5 + [1] * 3 + [2] * 3 + [3])
    assert hot_columns_oracle(colidx, 5, 128, 1) == (1, 5 / 12)
    assert hot_columns_oracle(colidx, 5, 64, 1) == (4, 1.0)
    assert hot_columns_oracle(colidx, 5, 100, 1) == (1, 5 / 12)  # 400-byte rows occupy 512 bytes of cache lines
    assert hot_columns_oracle(colidx, 5, 128, 2) == (4, 1.0)
    assert hot_columns_oracle(np.zeros(0, np.int64), 3, 64, 1) == (0, 0.0)
