"""Plain numpy statement of what the SpMM planner must produce (test infrastructure only).

The paper has no planner: it names load balancing and irregular access as the known SpMM
problems (related-work section) and leaves GPU execution to future work (Section 6).  The
plan is this build's own structure, so its "oracle" is simply its definition written out
with sorts, searches and Python loops, no parallel tricks:

  * row length  len_i = rowptr[i+1] - rowptr[i]
  * class       0 "short" (len <= LW), 1 "wave" (LW < len <= CH), 2 "block" (len > CH)
  * windows     row i has merge-path key  key_i = rowptr[i] + ALPHA*i  (strictly increasing);
                window w owns the rows with key in [w*BN, (w+1)*BN); win_row_start[w] is the
                first such row; there are NW = (nnz + ALPHA*m)//BN + 1 windows
  * win_stage   per window (first entry, number of entries) from the first to the last short row among its first
                64 rows, the number capped at STAGE_MAX = 320; (0, -1) when it has no short row
  * wave_rows   the class-1 row ids, ascending; wave_span their entry ranges (rowptr[i], rowptr[i+1])
  * items       for every class-2 row, ascending: its nnz range cut into pieces of at most BCH;
                a row cut into more than one piece gets consecutive partial-sum slots
  * split       (row, first_slot, pieces) for every row with more than one piece, ascending

parity unpinned against the paper (nothing there to pin to); pinned instead by the structural
invariants in tests/test_plan_oracle.py (every row is covered exactly once, pieces tile the
row's nnz range, windows partition the rows, bounds on rows and nnz per window).
"""
from __future__ import annotations

from typing import Dict

import numpy as np


def plan_oracle(rowptr: np.ndarray, BN: int, ALPHA: int, LW: int, CH: int, BCH: int) -> Dict[str, np.ndarray]:
    rp = np.asarray(rowptr, dtype=np.int64)
    m = rp.shape[0] - 1
    nnz = int(rp[-1]) if m >= 0 else 0
    lens = np.diff(rp)
    cls = np.where(lens <= LW, 0, np.where(lens <= CH, 1, 2)).astype(np.int32)

    NW = (nnz + ALPHA * m) // BN + 1
    key = rp[:m] + ALPHA * np.arange(m, dtype=np.int64)
    win_row_start = np.searchsorted(key, np.arange(NW + 1, dtype=np.int64) * BN, side="left").astype(np.int32)
    win_row_start[NW] = m

    STAGE_MAX, WINDOW_ROWS_MAX = 320, 64
    win_stage = np.zeros((NW, 2), dtype=np.int32)
    for w in range(NW):
        r0, r1 = int(win_row_start[w]), min(int(win_row_start[w + 1]), int(win_row_start[w]) + WINDOW_ROWS_MAX)
        short = [r for r in range(r0, r1) if cls[r] == 0]
        if short:
            beg, end = int(rp[short[0]]), int(rp[short[-1] + 1])
            win_stage[w] = (beg, min(end - beg, STAGE_MAX))
        else:
            win_stage[w] = (0, -1)

    wave_rows = np.nonzero(cls == 1)[0].astype(np.int32)

    items, split = [], []
    slot = 0
    for i in np.nonzero(cls == 2)[0]:
        p0, p1 = int(rp[i]), int(rp[i + 1])
        pieces = -(-(p1 - p0) // BCH)
        if pieces > 1:
            split.append((int(i), slot, pieces, 0))
        for c in range(pieces):
            a = p0 + c * BCH
            b = min(p1, a + BCH)
            items.append((int(i), a, b, slot + c if pieces > 1 else -1))
        if pieces > 1:
            slot += pieces
    return {
        "row_class": cls,
        "win_row_start": win_row_start,
        "win_stage": win_stage,
        "wave_rows": wave_rows,
        "wave_span": np.stack([rp[wave_rows], rp[wave_rows + 1]], axis=1).astype(np.int32).reshape(-1, 2),
        "items": np.array(items, dtype=np.int32).reshape(-1, 4),
        "split": np.array(split, dtype=np.int32).reshape(-1, 4),
        "n_slots": np.int64(slot),
        "n_short": np.int64(int((cls == 0).sum())),
    }


def hot_columns_oracle(colidx: np.ndarray, k: int, n: int, budget_kb: int):
    """Which columns of A the planner marks as hot (their rows of B keep the default cache policy), stated plainly:
    count how often every column occurs; put the counts into bins, 16 per power of two (bin 0: never occurs; a count x
    with highest set bit e falls into bin 16 e + (the four bits below the highest) + 1); take whole bins from the
    largest counts downwards while their columns, at one row of B rounded up to 128-byte lines each, fit budget_kb KB.
    Returns (number of hot columns, share of the stored entries that point at them).  No counterpart in the paper:
    parity unpinned against it, like the rest of the plan; results never depend on the marking."""
    deg = np.bincount(np.asarray(colidx, dtype=np.int64), minlength=k)

    def degree_bin(x: int) -> int:
        if x <= 0:
            return 0
        e = int(x).bit_length() - 1
        frac = (x >> (e - 4)) & 15 if e >= 4 else (x << (4 - e)) & 15
        return e * 16 + frac + 1

    bins = np.array([degree_bin(int(x)) for x in deg])
    max_rows = max(1, budget_kb * 1024 // (((n * 4 + 127) // 128) * 128))
    rows, entries = 0, 0
    for b in range(int(bins.max()) if len(bins) else 0, 0, -1):
        cnt = int((bins == b).sum())
        if rows + cnt > max_rows:
            break
        rows += cnt
        entries += int(deg[bins == b].sum())
    return rows, (entries / len(colidx) if len(colidx) else 0.0)


def coo_rowptr_oracle(m: int, row_idx: np.ndarray) -> np.ndarray:
    """Row pointers of a coordinate list (paper, Appendix C, coordinate format) whose entries are sorted by row:
    rowptr[i] = number of entries with row < i, i.e. the running sum of the per-row counts."""
    counts = np.bincount(np.asarray(row_idx, dtype=np.int64), minlength=m)
    out = np.zeros(m + 1, dtype=np.int64)
    np.cumsum(counts, out=out[1:])
    return out.astype(np.int32)


def dcsr_rowptr_oracle(m: int, row_ids: np.ndarray, row_pos: np.ndarray) -> np.ndarray:
    """CSR row pointers of a doubly compressed matrix (paper, Appendix C): row row_ids[r] holds the entries
    [row_pos[r], row_pos[r+1]); every other row is empty.  Written as per-row lengths and their running sum."""
    lens = np.zeros(m, dtype=np.int64)
    lens[np.asarray(row_ids, dtype=np.int64)] = np.diff(np.asarray(row_pos, dtype=np.int64))
    out = np.zeros(m + 1, dtype=np.int64)
    np.cumsum(lens, out=out[1:])
    return out.astype(np.int32)
