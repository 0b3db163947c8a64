"""Seeded generators for the five SpMM workloads and for small/edge-case operands.

Every array is a pure function of (generator arguments, seed): random streams are
numpy Philox generators keyed by (seed, stream id), so a problem can be rebuilt
identically on any machine.  All CSR matrices leave here with int32 ``rowptr`` /
``colidx`` (sorted and duplicate-free inside a row unless a caller asks otherwise)
and fp32 ``vals``; B is fp32, row-major, with row stride ``ldb >= n``.

The paper measures SpMM on public sparse-matrix and graph collections multiplied by a
random dense matrix (Section 5.4 and Appendix E.1; GCN on citation graphs with hidden
size 128, Section 5.1 and Table 1).  None of those files is used here: the generators
only reproduce sizes, density and degree shape with synthetic draws.

Nothing in this module multiplies A by B.
"""
from __future__ import annotations

import dataclasses
import math
import os
from typing import Dict, Optional

import numpy as np

CONFIG_NAMES = {
    1: "tiny_powerlaw_4096_n64",
    2: "uniform_1pct_16384_n128",
    3: "gcn_mid_169343_n128",
    4: "large_powerlaw_2449029_n100",
    5: "pruned_ffn_4096x16384_n2048",
}


@dataclasses.dataclass
class SpmmProblem:
    """Operands of one SpMM call, as host numpy arrays."""

    name: str
    m: int
    k: int
    n: int
    rowptr: np.ndarray  # int32 [m+1]
    colidx: np.ndarray  # int32 [nnz]
    vals: np.ndarray  # float32 [nnz]
    B: np.ndarray  # float32 [k, ldb]; columns n..ldb-1 are padding
    meta: Dict[str, object] = dataclasses.field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    @property
    def ldb(self) -> int:
        return int(self.B.shape[1]) if self.B.ndim == 2 else self.n

    @property
    def row_lengths(self) -> np.ndarray:
        return np.diff(self.rowptr.astype(np.int64))

    def check(self) -> None:
        """Structural validity (what a caller of the library must guarantee)."""
        assert self.rowptr.dtype == np.int32 and self.colidx.dtype == np.int32
        assert self.vals.dtype == np.float32 and self.B.dtype == np.float32
        assert self.rowptr.shape == (self.m + 1,)
        assert int(self.rowptr[0]) == 0
        assert np.all(np.diff(self.rowptr.astype(np.int64)) >= 0)
        assert self.colidx.shape == (self.nnz,) and self.vals.shape == (self.nnz,)
        if self.nnz:
            assert int(self.colidx.min()) >= 0 and int(self.colidx.max()) < self.k
        assert self.B.shape[0] == self.k and self.B.shape[1] >= self.n


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([int(seed), int(stream)])))


def _normal_f32(rng: np.random.Generator, rows: int, cols: int) -> np.ndarray:
    out = np.empty((rows, cols), dtype=np.float32)
    step = max(1, (1 << 24) // max(cols, 1))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        out[r0:r1] = rng.standard_normal((r1 - r0, cols), dtype=np.float32)
    return out


def _rowptr_from_lengths(lens: np.ndarray) -> np.ndarray:
    rp = np.zeros(lens.shape[0] + 1, dtype=np.int64)
    np.cumsum(lens, out=rp[1:])
    if rp[-1] >= 2**31:
        raise ValueError("nnz does not fit int32")
    return rp.astype(np.int32)


# --------------------------------------------------------------------------------------
# config 1: tiny directed power-law graph
# --------------------------------------------------------------------------------------
def tiny_powerlaw(m: int = 4096, n: int = 64, seed: int = 0, alpha: float = 2.0, dmax: int = 64) -> SpmmProblem:
    """Square directed graph; out-degree ~ Zipf(alpha) truncated to [1, dmax]; plus self-loops.

    vals[p] = 1/sqrt(deg_i * deg_j) with deg_x the stored length of row x (self-loop included).
    """
    k = m
    rng = _rng(seed, 11)
    d = np.arange(1, dmax + 1, dtype=np.float64)
    pmf = d ** (-alpha)
    pmf /= pmf.sum()
    deg = rng.choice(np.arange(1, dmax + 1), size=m, p=pmf)
    deg = np.minimum(deg, k - 1)
    cols = []
    for i in range(m):
        t = rng.choice(k - 1, size=int(deg[i]), replace=False)
        t = t + (t >= i)  # skip the diagonal, it is added explicitly
        row = np.concatenate([t, [i]])
        row.sort()
        cols.append(row)
    lens = np.array([c.shape[0] for c in cols], dtype=np.int64)
    rowptr = _rowptr_from_lengths(lens)
    colidx = np.concatenate(cols).astype(np.int32)
    rows_of = np.repeat(np.arange(m), lens)
    vals = (1.0 / np.sqrt(lens[rows_of].astype(np.float64) * lens[colidx].astype(np.float64))).astype(np.float32)
    B = _normal_f32(_rng(seed, 12), k, n)
    return SpmmProblem("tiny_powerlaw", m, k, n, rowptr, colidx, vals, B,
                       {"alpha": alpha, "dmax": dmax, "seed": seed})


# --------------------------------------------------------------------------------------
# config 2: uniform random, fixed row length, columns without replacement
# --------------------------------------------------------------------------------------
def _distinct_columns(rng: np.random.Generator, rows: int, k: int, per_row: int) -> np.ndarray:
    """rows x per_row distinct uniform columns per row, each row sorted ascending."""
    if per_row > k:
        raise ValueError("per_row > k")
    if rows * k <= (1 << 24) or per_row * 4 > k:
        keys = rng.random((rows, k))
        sel = np.argpartition(keys, per_row - 1, axis=1)[:, :per_row] if per_row < k else np.tile(np.arange(k), (rows, 1))
        sel.sort(axis=1)
        return sel.astype(np.int64)
    extra = per_row + max(16, int(4 * per_row * per_row / k) + 16)
    cand = rng.integers(0, k, size=(rows, extra), dtype=np.int64)
    order = np.argsort(cand, axis=1, kind="stable")
    srt = np.take_along_axis(cand, order, axis=1)
    dup_sorted = np.zeros_like(srt, dtype=bool)
    dup_sorted[:, 1:] = srt[:, 1:] == srt[:, :-1]
    dup = np.zeros_like(dup_sorted)
    np.put_along_axis(dup, order, dup_sorted, axis=1)
    keep = ~dup
    rank = np.cumsum(keep, axis=1)
    keep &= rank <= per_row
    out = np.empty((rows, per_row), dtype=np.int64)
    good = keep.sum(axis=1) == per_row
    out[good] = cand[good][keep[good]].reshape(-1, per_row)
    for r in np.nonzero(~good)[0]:  # practically never taken
        out[r] = rng.choice(k, size=per_row, replace=False)
    out.sort(axis=1)
    return out


def uniform_rows(m: int = 16384, k: int = 16384, density: float = 0.01, n: int = 128, seed: int = 0) -> SpmmProblem:
    """Every row has round(density*k) distinct uniform columns; vals ~ U(-1,1)."""
    per_row = max(1, int(round(density * k)))
    rng = _rng(seed, 21)
    blocks = []
    step = max(1, (1 << 22) // max(per_row, 1))
    for r0 in range(0, m, step):
        blocks.append(_distinct_columns(rng, min(step, m - r0), k, per_row))
    cols = np.concatenate(blocks, axis=0)
    rowptr = _rowptr_from_lengths(np.full(m, per_row, dtype=np.int64))
    colidx = cols.reshape(-1).astype(np.int32)
    vals = _rng(seed, 22).uniform(-1.0, 1.0, size=colidx.shape[0]).astype(np.float32)
    B = _normal_f32(_rng(seed, 23), k, n)
    return SpmmProblem("uniform_rows", m, k, n, rowptr, colidx, vals, B,
                       {"density": density, "per_row": per_row, "seed": seed})


# --------------------------------------------------------------------------------------
# configs 3 and 4: symmetric Chung-Lu power-law graph
# --------------------------------------------------------------------------------------
def _rank_density_params(N: int, S: float, wmax: float, gamma: float):
    """Endpoint density over ranks x in [0,N): proportional to (x+r0)^(-a), a = 1/(gamma-1).

    Node r owns [r, r+1), so its expected degree is w_r = S * P(r).  r0 is found by bisection
    such that the heaviest node has w_0 = wmax.
    """
    a = 1.0 / (gamma - 1.0)
    e = 1.0 - a

    def w0(r0):
        lo, hi = r0 ** e, (N + r0) ** e
        return S * (((1.0 + r0) ** e - lo) / (hi - lo))

    lo_r, hi_r = 1e-9, float(N) * 64
    if w0(lo_r) < wmax:
        return a, e, lo_r
    for _ in range(200):
        mid = math.sqrt(lo_r * hi_r)
        if w0(mid) > wmax:
            lo_r = mid
        else:
            hi_r = mid
    return a, e, math.sqrt(lo_r * hi_r)


def chung_lu_graph(N: int, mean_degree: float, wmax: float, gamma: float, n: int, *, normalize: str,
                   self_loops: bool, seed: int = 0, relabel: bool = True, name: str = "chung_lu") -> SpmmProblem:
    """Undirected Chung-Lu graph with power-law expected degrees, stored as a symmetric CSR.

    ``normalize='sym'``: vals = 1/sqrt(d_i d_j), d = stored row length (D^-1/2 (A+I) D^-1/2 when
    self_loops).  ``normalize='row'``: vals = 1/d_i (D^-1 A).  Nodes get a seeded random relabelling
    so that degree is uncorrelated with the row index.
    """
    S = float(N) * mean_degree  # number of endpoint draws = 2 * (#sampled undirected edges)
    E = int(round(S / 2))
    a, e, r0 = _rank_density_params(N, S, wmax, gamma)
    lo, hi = r0 ** e, (N + r0) ** e
    rng = _rng(seed, 31)

    def draw(count):
        out = np.empty(count, dtype=np.int64)
        step = 1 << 24
        for s0 in range(0, count, step):
            u = rng.random(min(step, count - s0))
            x = (u * (hi - lo) + lo) ** (1.0 / e) - r0
            out[s0:s0 + u.shape[0]] = np.clip(x.astype(np.int64), 0, N - 1)
        return out

    u = draw(E)
    v = draw(E)
    if relabel:
        perm = _rng(seed, 32).permutation(N).astype(np.int64)
        u = perm[u]
        v = perm[v]
    keep = u != v
    u, v = u[keep], v[keep]
    parts = [u * N + v, v * N + u]
    del u, v, keep
    if self_loops:
        d = np.arange(N, dtype=np.int64)
        parts.append(d * N + d)
    keys = np.concatenate(parts)
    del parts
    keys = np.unique(keys)  # sorts by (row, col) and removes multi-edges
    rows = keys // N
    cols = (keys - rows * N).astype(np.int32)
    del keys
    lens = np.bincount(rows, minlength=N).astype(np.int64)
    rowptr = _rowptr_from_lengths(lens)
    if normalize == "sym":
        dinv = np.zeros(N, dtype=np.float64)
        nz = lens > 0
        dinv[nz] = 1.0 / np.sqrt(lens[nz].astype(np.float64))
        vals = (dinv[rows] * dinv[cols]).astype(np.float32)
    elif normalize == "row":
        vals = (1.0 / lens[rows].astype(np.float64)).astype(np.float32)
    else:
        raise ValueError(normalize)
    del rows
    B = _normal_f32(_rng(seed, 33), N, n)
    return SpmmProblem(name, N, N, n, rowptr, cols, vals, B,
                       {"mean_degree": mean_degree, "wmax": wmax, "gamma": gamma, "r0": r0,
                        "normalize": normalize, "self_loops": self_loops, "seed": seed, "relabel": relabel})


# --------------------------------------------------------------------------------------
# config 5: unstructured-pruned weight times activations
# --------------------------------------------------------------------------------------
def pruned_weight(m: int = 4096, k: int = 16384, sparsity: float = 0.9, n: int = 2048, seed: int = 0,
                  std: float = 0.02) -> SpmmProblem:
    """Bernoulli(1-sparsity) mask over an m x k weight; kept vals ~ N(0, std); B = activations ~ N(0,1)."""
    rng = _rng(seed, 41)
    keep_p = 1.0 - sparsity
    cols, lens = [], np.zeros(m, dtype=np.int64)
    step = max(1, (1 << 22) // max(k, 1))
    for r0 in range(0, m, step):
        r1 = min(m, r0 + step)
        mask = rng.random((r1 - r0, k)) < keep_p
        rr, cc = np.nonzero(mask)
        lens[r0:r1] = np.bincount(rr, minlength=r1 - r0)
        cols.append(cc.astype(np.int32))
    colidx = np.concatenate(cols) if cols else np.zeros(0, np.int32)
    rowptr = _rowptr_from_lengths(lens)
    vals = (_rng(seed, 42).standard_normal(colidx.shape[0]) * std).astype(np.float32)
    B = _normal_f32(_rng(seed, 43), k, n)
    return SpmmProblem("pruned_weight", m, k, n, rowptr, colidx, vals, B,
                       {"sparsity": sparsity, "std": std, "seed": seed})


# --------------------------------------------------------------------------------------
# generic pattern builder for edge cases
# --------------------------------------------------------------------------------------
def csr_from_row_lengths(lens, k: int, n: int, seed: int = 0, *, sorted_cols: bool = True,
                         duplicates: bool = False, ldb: Optional[int] = None,
                         name: str = "custom") -> SpmmProblem:
    """CSR with prescribed row lengths.  Columns uniform; distinct per row unless ``duplicates``.

    ``sorted_cols=False`` leaves every row in draw order (unsorted); ``duplicates=True`` draws
    with replacement so a row may store the same column several times.
    """
    lens = np.asarray(lens, dtype=np.int64)
    m = lens.shape[0]
    rng = _rng(seed, 51)
    cols = []
    for L in lens:
        L = int(L)
        if duplicates or L > k:
            c = rng.integers(0, k, size=L, dtype=np.int64)
        else:
            c = rng.choice(k, size=L, replace=False)
        if sorted_cols:
            c = np.sort(c)
        cols.append(c)
    colidx = (np.concatenate(cols) if m and lens.sum() else np.zeros(0)).astype(np.int32)
    rowptr = _rowptr_from_lengths(lens)
    vals = _rng(seed, 52).uniform(-1.0, 1.0, size=colidx.shape[0]).astype(np.float32)
    B = _normal_f32(_rng(seed, 53), k, n)
    p = SpmmProblem(name, m, k, n, rowptr, colidx, vals, B, {"seed": seed})
    return with_padding(p, ldb) if ldb is not None and ldb != n else p


def integer_valued(p: SpmmProblem, seed: int = 0) -> SpmmProblem:
    """Same sparsity pattern, vals in {-4..4}\\{0}, B in {-8..8}: every partial sum is a small integer."""
    rng = _rng(seed, 61)
    mag = rng.integers(1, 5, size=p.nnz)
    sgn = rng.integers(0, 2, size=p.nnz) * 2 - 1
    vals = (mag * sgn).astype(np.float32)
    B = np.full(p.B.shape, np.nan, dtype=np.float32) if p.ldb != p.n else np.empty(p.B.shape, np.float32)
    B[:, :p.n] = _rng(seed, 62).integers(-8, 9, size=(p.k, p.n)).astype(np.float32)
    return SpmmProblem(p.name + "_int", p.m, p.k, p.n, p.rowptr, p.colidx, vals, B, dict(p.meta, integer=True))


def with_padding(p: SpmmProblem, ldb: int, fill: float = float("nan")) -> SpmmProblem:
    """Copy of the problem whose B has row stride ``ldb > n``; padding columns hold ``fill``."""
    assert ldb >= p.n
    B = np.full((p.k, ldb), fill, dtype=np.float32)
    B[:, :p.n] = p.B[:, :p.n]
    return SpmmProblem(p.name, p.m, p.k, p.n, p.rowptr, p.colidx, p.vals, B, dict(p.meta, ldb=ldb))


def count_unique_columns(p: SpmmProblem) -> int:
    if p.nnz == 0:
        return 0
    seen = np.zeros(p.k, dtype=bool)
    seen[p.colidx] = True
    return int(seen.sum())


def min_traffic_bytes(p: SpmmProblem) -> int:
    """Minimum HBM traffic of one SpMM: A streamed once, rowptr, C written once, each touched B row read once."""
    return p.nnz * 8 + (p.m + 1) * 4 + p.m * p.n * 4 + count_unique_columns(p) * p.n * 4


# --------------------------------------------------------------------------------------
# the five named workloads
# --------------------------------------------------------------------------------------
def make_scaled_config(cfg: int, scale: float = 1.0, seed: int = 0) -> SpmmProblem:
    """Workload ``cfg`` (1..5) with its row/column counts multiplied by ``scale`` (n unchanged)."""
    s = float(scale)

    def sz(x, lo=8):
        return max(lo, int(round(x * s)))

    if cfg == 1:
        p = tiny_powerlaw(m=sz(4096, 80), n=64, seed=seed)
    elif cfg == 2:
        p = uniform_rows(m=sz(16384), k=sz(16384, 200), density=0.01, n=128, seed=seed)
    elif cfg == 3:
        N = sz(169343, 64)
        p = chung_lu_graph(N, 14.8, min(1.7e4, N / 4), 2.1, 128, normalize="sym", self_loops=True,
                           seed=seed, name="gcn_mid")
    elif cfg == 4:
        N = sz(2449029, 64)
        S = N * 50.2
        p = chung_lu_graph(N, 50.2, min(math.sqrt(S), N / 4), 2.1, 100, normalize="row", self_loops=False,
                           seed=seed, name="large_powerlaw")
    elif cfg == 5:
        p = pruned_weight(m=sz(4096), k=sz(16384, 64), sparsity=0.9, n=2048 if s >= 1.0 else max(256, int(2048 * s) // 4 * 4), seed=seed)
    else:
        raise ValueError("cfg must be 1..5")
    p.meta["config"] = cfg
    p.meta["scale"] = s
    p.name = CONFIG_NAMES[cfg] if s == 1.0 else f"{CONFIG_NAMES[cfg]}_x{s:g}"
    return p


def make_config(cfg: int, seed: int = 0, cache_dir: Optional[str] = None) -> SpmmProblem:
    """Full-size workload ``cfg``.  With ``cache_dir`` (or $SCORCH_WORKLOAD_CACHE) the arrays are kept on disk."""
    cache_dir = cache_dir if cache_dir is not None else os.environ.get("SCORCH_WORKLOAD_CACHE")
    path = None
    if cache_dir:
        os.makedirs(cache_dir, exist_ok=True)
        path = os.path.join(cache_dir, f"spmm_cfg{cfg}_seed{seed}.npz")
        if os.path.exists(path):
            with np.load(path, allow_pickle=False) as z:
                p = SpmmProblem(CONFIG_NAMES[cfg], int(z["m"]), int(z["k"]), int(z["n"]),
                                z["rowptr"], z["colidx"], z["vals"], z["B"], {"config": cfg, "seed": seed, "scale": 1.0})
            return p
    p = make_scaled_config(cfg, 1.0, seed)
    if path:
        tmp = path + f".tmp{os.getpid()}.npz"
        np.savez(tmp, m=p.m, k=p.k, n=p.n, rowptr=p.rowptr, colidx=p.colidx, vals=p.vals, B=p.B)
        os.replace(tmp, path)
    return p
