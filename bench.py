#!/usr/bin/env python3
"""Benchmark of the CSR SpMM hot path on one MI355X.

One "step" = one planned SpMM (C = A.B) over one resident synthetic workload: the fused
execution launch plus, when rows were split across workgroups, the small fix-up launch.
The plan is built once, outside the timed region, and its time is reported separately.

Prints ONE JSON line.  `value` is GFLOP/s = 2*nnz*n / t (the metric of the workloads);
`roofline` prices the step against the minimum HBM traffic
    nnz*8 (colidx+vals) + (m+1)*4 (rowptr) + m*n*4 (C written) + U*n*4 (distinct B rows read)
at MI355X's 8 TB/s; `cpu_baseline` is the serial fp64 oracle timed on a bounded row sample
of the same workload (the GPU result is then compared with the oracle on every row, outside the timed parts).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PLAIN_FMA_TFLOPS = 78.6  # fp32 vector rate without packed operations: 256 CUs x 64 lanes x 2 flop x 2.4 GHz
HEADLINE_CONFIG = 4  # large power-law graph aggregation: the largest single-GPU workload, HBM-bound


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def load_traffic_table():
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE), if committed."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(path):
        with open(path) as f:
            return json.load(f)
    return {}


class Resident:
    """A workload uploaded to the GPU with its plan."""

    def __init__(self, p, torch, sp):
        self.p = p
        dev = torch.device("cuda:0")
        self.rowptr = torch.from_numpy(p.rowptr).to(dev)
        self.colidx = torch.from_numpy(p.colidx).to(dev)
        self.vals = torch.from_numpy(p.vals).to(dev)
        self.B = torch.from_numpy(p.B).to(dev)
        self.C = torch.empty((p.m, p.n), dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        self.plan = sp.scorch_spmm_plan(p.m, p.k, p.n, self.rowptr, p.nnz, colidx=self.colidx)
        self.plan_ms = (time.perf_counter() - t0) * 1e3
        self.sp = sp

    def step(self):
        self.sp.scorch_spmm_csr_planned(self.plan, self.rowptr, self.colidx, self.vals, self.B, self.C)


def time_steps(res, torch, steps, warmup, flush=None):
    """Wall-clock over `steps` back-to-back steps, plus HIP-event time of every step on the launch stream."""
    for _ in range(warmup):
        res.step()
    torch.cuda.synchronize()
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        if flush is not None:
            flush()
        starts[i].record()
        res.step()
        stops[i].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    ev = np.array([starts[i].elapsed_time(stops[i]) for i in range(steps)])
    return wall_ms, ev


def summarize(p, wall_ms, ev_ms, bytes_min):
    t = float(np.mean(ev_ms)) * 1e-3
    return {
        "gflops": 2.0 * p.nnz * p.n / t / 1e9,
        "gbs_min_traffic": bytes_min / t / 1e9,
        "frac_hbm": bytes_min / t / 1e9 / HBM_PEAK_GBS,
        "event_ms_mean": float(np.mean(ev_ms)),
        "event_ms_median": float(np.median(ev_ms)),
        "event_ms_min": float(np.min(ev_ms)),
        "wall_ms_per_step": wall_ms,
    }


def time_sddmm(res, torch, sp, d, steps=30, warmup=5):
    """SDDMM (D = A (.) (B C)) on the resident pattern with random m x d and k x d factors: events per call."""
    p = res.p
    g = torch.Generator(device="cuda:0").manual_seed(1)
    X = torch.randn((p.m, d), generator=g, dtype=torch.float32, device="cuda:0")
    Yt = torch.randn((p.k, d), generator=g, dtype=torch.float32, device="cuda:0")
    out = torch.empty(max(p.nnz, 1), dtype=torch.float32, device="cuda:0")

    def call():
        sp.scorch_sddmm_csr_planned(res.plan, d, res.rowptr, res.colidx, res.vals, X, Yt, out)

    for _ in range(warmup):
        call()
    torch.cuda.synchronize()
    ev = []
    for _ in range(steps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        call()
        b.record()
        ev.append((a, b))
    torch.cuda.synchronize()
    ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
    uniq = int(np.count_nonzero(np.bincount(p.colidx, minlength=p.k))) if p.nnz else 0
    bytes_min = p.nnz * 12 + (p.m + 1) * 4 + p.m * d * 4 + uniq * d * 4
    return {"d": d, "event_ms_mean": ms, "gflops": 2.0 * p.nnz * d / (ms * 1e-3) / 1e9,
            "bytes_min": bytes_min, "gbs_min_traffic": bytes_min / (ms * 1e-3) / 1e9,
            "frac_hbm": bytes_min / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}


def _event_ms(torch, call, steps, warmup):
    for _ in range(warmup):
        call()
    torch.cuda.synchronize()
    ev = []
    for _ in range(steps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        call()
        b.record()
        ev.append((a, b))
    torch.cuda.synchronize()
    return float(np.mean([a.elapsed_time(b) for a, b in ev]))


def time_widenings(res, torch, sp, steps=30, warmup=5):
    """Short timings, on the resident pattern, of the paths built around the SpMM: SpMV (n = 1, its own plan), the
    fused bias + ReLU epilogue (against the same call without it), and the row-pointer build from a coordinate list
    and from doubly compressed rows.  Bytes are the minimum-traffic model of each call."""
    p = res.p
    dev = "cuda:0"
    out = {}
    g = torch.Generator(device=dev).manual_seed(2)
    # SpMV: y = A x
    x = torch.randn((p.k, 1), generator=g, dtype=torch.float32, device=dev)
    y = torch.empty((p.m, 1), dtype=torch.float32, device=dev)
    plan1 = sp.scorch_spmm_plan(p.m, p.k, 1, res.rowptr, p.nnz, colidx=res.colidx)
    ms = _event_ms(torch, lambda: sp.scorch_spmm_csr_planned(plan1, res.rowptr, res.colidx, res.vals, x, y), steps, warmup)
    ms_graph = time_graph_replay(res, torch, sp, call=lambda st: sp.scorch_spmm_csr_planned(plan1, res.rowptr, res.colidx,
                                                                                             res.vals, x, y, stream=st))
    plan1.destroy()
    uniq = int(np.count_nonzero(np.bincount(p.colidx, minlength=p.k))) if p.nnz else 0
    b = p.nnz * 8 + (p.m + 1) * 4 + p.m * 4 + uniq * 4
    out["spmv"] = {"event_ms_mean": ms, "graph_replay_ms_per_step": ms_graph, "gflops": 2.0 * p.nnz / (ms * 1e-3) / 1e9,
                   "bytes_min": b, "frac_hbm": b / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                   "frac_hbm_in_a_graph": b / (ms_graph * 1e-3) / 1e9 / HBM_PEAK_GBS}
    # fused epilogue: C = relu(A B + bias)
    bias = torch.randn(p.n, generator=g, dtype=torch.float32, device=dev)
    ms_e = _event_ms(torch, lambda: sp.scorch_spmm_csr_planned_epilogue(res.plan, res.rowptr, res.colidx, res.vals, res.B,
                                                                         bias, 1, res.C), steps, warmup)
    ms_p = _event_ms(torch, res.step, steps, warmup)

    def unfused():
        res.step()
        res.C.add_(bias).relu_()
    ms_u = _event_ms(torch, unfused, steps, warmup)
    out["epilogue"] = {"fused_event_ms_mean": ms_e, "plain_spmm_event_ms_mean": ms_p,
                       "spmm_then_elementwise_event_ms_mean": ms_u}
    # one graph-convolution layer relu(A (H W) + b), hidden width n -> n (square patterns only): dense product in the
    # dense library, aggregation + bias + activation in one planned call
    if p.m == p.k:
        from paper_2405_16883_amd.gcn import GcnLayer
        layer = GcnLayer(p.m, res.rowptr, res.colidx, res.vals, p.nnz)
        H = torch.randn((p.m, p.n), generator=g, dtype=torch.float32, device=dev)
        W = torch.randn((p.n, p.n), generator=g, dtype=torch.float32, device=dev) * 0.05
        ms_l = _event_ms(torch, lambda: layer.forward(H, W, bias, relu=True), steps, warmup)
        ms_mm = _event_ms(torch, lambda: torch.mm(H, W), steps, warmup)
        layer.close()
        out["gcn_layer"] = {"width": int(p.n), "event_ms_mean": ms_l, "dense_product_event_ms_mean": ms_mm}
    # second storage formats: row pointers from sorted row coordinates / from the list of stored rows
    rows = torch.repeat_interleave(torch.arange(p.m, dtype=torch.int32, device=dev),
                                   (res.rowptr[1:] - res.rowptr[:-1]).long())
    rp = torch.empty(p.m + 1, dtype=torch.int32, device=dev)
    ms_c = _event_ms(torch, lambda: sp.scorch_coo_to_csr_rowptr(p.m, rows, rp), steps, warmup)
    ok_c = bool(torch.equal(rp, res.rowptr))
    lens = res.rowptr[1:] - res.rowptr[:-1]
    ids = torch.nonzero(lens > 0).flatten().to(torch.int32)
    pos = torch.cat([res.rowptr[:-1][ids.long()], res.rowptr[-1:]]).to(torch.int32)
    ms_d = _event_ms(torch, lambda: sp.scorch_dcsr_to_csr_rowptr(p.m, ids, pos, rp), steps, warmup)
    ok_d = bool(torch.equal(rp, res.rowptr))
    bc = p.nnz * 4 + (p.m + 1) * 4
    out["formats"] = {"coo_rowptr_event_ms_mean": ms_c, "coo_frac_hbm": bc / (ms_c * 1e-3) / 1e9 / HBM_PEAK_GBS,
                      "coo_matches_rowptr": ok_c, "dcsr_rowptr_event_ms_mean": ms_d, "dcsr_matches_rowptr": ok_d}
    return out


def time_graph_replay(res, torch, sp, steps_per_graph=20, replays=10, call=None):
    """Per-step time when `steps_per_graph` planned calls are recorded into one HIP graph (launch overhead amortised).
    `call(stream)` issues one step (default: the resident workload's planned SpMM)."""
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    if call is None:
        def call(stream):
            sp.scorch_spmm_csr_planned(res.plan, res.rowptr, res.colidx, res.vals, res.B, res.C, stream=stream)
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for _ in range(steps_per_graph):
                call(side)
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(replays):
        graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / (replays * steps_per_graph)


def measure_practical_peak(torch, flush_buf):
    """What this chip delivers, measured now, on the launch stream, to the access patterns an SpMM consists of:
    a streaming read, a copy, and random gathers of whole 256/400/512-byte rows from tables that fit one die's L2 (2 MB),
    that are two and four times one L2 (8 and 16 MB: about half and a quarter of the gathers hit L2, the mix a graph
    workload sees), that fit the 256 MB memory-side cache (96 MB) and that exceed both (2 GiB).  GB/s of useful bytes, best of 3 launches.
    The probe kernels live in a library of their own (paper_2405_16883_amd/csrc/probes), not in the product."""
    import ctypes

    from paper_2405_16883_amd.build import PROBES_LIB_PATH, build_probes
    if not os.path.exists(PROBES_LIB_PATH):
        log(f"[bench] {PROBES_LIB_PATH} is missing: building the bandwidth probes")
        build_probes()
    lib = ctypes.CDLL(PROBES_LIB_PATH)
    vp, i32, i64, u32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32, ctypes.c_size_t
    lib.scorch_probe_stream_read.argtypes = [vp, sz, i32, vp, vp]
    lib.scorch_probe_copy.argtypes = [vp, vp, sz, vp]
    lib.scorch_probe_row_gather.argtypes = [vp, u32, u32, i32, i64, i32, vp, vp]
    lib.scorch_probe_lds_read.argtypes = [i32, i32, vp, vp]
    dev = "cuda:0"
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    sink = torch.zeros(64, dtype=torch.float32, device=dev)
    big = torch.zeros(1 << 29, dtype=torch.float32, device=dev)  # 2 GiB table / copy destination

    def best_ms(call, reps=3):
        call()
        torch.cuda.synchronize()
        out = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            rc = call()
            b.record()
            torch.cuda.synchronize()
            assert rc == 0, "probe launch failed"
            out.append(a.elapsed_time(b))
        return min(out)

    gib = 1 << 30
    pk = {"unit": "GB/s of useful bytes", "hbm_spec_gbs": HBM_PEAK_GBS}
    ms = best_ms(lambda: lib.scorch_probe_stream_read(big.data_ptr(), 2 * gib, 1, sink.data_ptr(), stream))
    pk["stream_read_2GiB"] = 2 * gib / ms / 1e6
    ms = best_ms(lambda: lib.scorch_probe_copy(flush_buf.data_ptr(), big.data_ptr(), gib, stream))
    pk["copy_1GiB_read_plus_write"] = 2 * gib / ms / 1e6
    lds_blocks, lds_iters = 256 * 8, 4096
    ms = best_ms(lambda: lib.scorch_probe_lds_read(lds_blocks, lds_iters, sink.data_ptr(), stream))
    pk["lds_read_b128"] = lds_blocks * 1024 * lds_iters * 16 / ms / 1e6
    groups, iters = 65536, 256
    pk["row_gather"] = {}
    for row_floats in (64, 100, 128):
        row = {}
        for label, table_bytes in (("table_2MB_fits_one_L2", 2 << 20), ("table_8MB_twice_one_L2", 8 << 20),
                                   ("table_16MB_four_times_one_L2", 16 << 20),
                                   ("table_96MB_fits_memory_side_cache", 96 << 20), ("table_2GiB_beyond_both", 2 * gib)):
            rows = table_bytes // (row_floats * 4)
            ms = best_ms(lambda: lib.scorch_probe_row_gather(big.data_ptr(), rows, row_floats, row_floats, groups, iters,
                                                             sink.data_ptr(), stream))
            row[label] = groups * iters * row_floats * 4 / ms / 1e6
        pk["row_gather"][f"{row_floats * 4}B_rows"] = row
    del big
    torch.cuda.empty_cache()
    return pk


def practical_floor(p, bytes_min, uniq_cols, pk, l2_hit_rate=None):
    """Time a kernel would need that streams A and C at the measured streaming-read rate and fetches one whole row of B
    per stored entry at the measured random-row-gather rate for rows of this width from a table of B's size (no reuse
    of a row between entries: what a graph without locality offers beyond its hub rows).  Returned with its inputs."""
    row_bytes = p.n * 4
    width = "256B_rows" if row_bytes <= 256 else ("400B_rows" if row_bytes <= 400 else "512B_rows")
    b_bytes = p.k * row_bytes
    size = ("table_2MB_fits_one_L2" if b_bytes <= (3 << 20) else
            "table_96MB_fits_memory_side_cache" if b_bytes <= (200 << 20) else "table_2GiB_beyond_both")
    gather_gbs = pk["row_gather"][width][size]
    stream_bytes = bytes_min - uniq_cols * row_bytes
    t = stream_bytes / (pk["stream_read_2GiB"] * 1e9) + p.nnz * row_bytes / (gather_gbs * 1e9)
    out = {"seconds": t, "gather_rate_used": f"{width}/{size}", "gather_gbs": gather_gbs,
           "gather_bytes": p.nnz * row_bytes, "streamed_bytes": stream_bytes}
    if l2_hit_rate is not None and size != "table_2MB_fits_one_L2":
        # The same at the share of L2 hits the counters report for this kernel (profiles/).  B inside the memory-side
        # cache: the gather rate is read off the probe's own mixes (tables of 1, 2, 4 and 24 times one die's L2, i.e.
        # about 100, 50, 25 and 4 % of L2 hits, misses served by the memory-side cache), linearly between the points.
        # B beyond it: no probe table mixes L2 hits with HBM-served misses, so hits are priced at the L2-resident rate
        # and misses at the beyond-both rate, one after the other (a model, pessimistic where the two overlap).
        h = float(l2_hit_rate)
        g = p.nnz * row_bytes
        rg = pk["row_gather"][width]
        if size == "table_96MB_fits_memory_side_cache":
            pts = [(0.04, rg["table_96MB_fits_memory_side_cache"]), (0.25, rg["table_16MB_four_times_one_L2"]),
                   (0.5, rg["table_8MB_twice_one_L2"]), (1.0, rg["table_2MB_fits_one_L2"])]
            hh = min(max(h, pts[0][0]), 1.0)
            for (h0, r0), (h1, r1) in zip(pts[:-1], pts[1:]):
                if hh <= h1:
                    rate = r0 + (r1 - r0) * (hh - h0) / (h1 - h0)
                    break
            t_g = g / (rate * 1e9)
            out["gather_gbs_at_measured_l2_hit_rate"] = rate
            out["l2_hit_model"] = "interpolated between the probe's tables of 1x, 2x, 4x and 24x one L2"
        else:
            t_g = g * h / (rg["table_2MB_fits_one_L2"] * 1e9) + g * (1.0 - h) / (gather_gbs * 1e9)
            out["l2_hit_model"] = "hits at the L2-resident rate, then misses at the beyond-both rate"
        out["seconds_at_measured_l2_hit_rate"] = stream_bytes / (pk["stream_read_2GiB"] * 1e9) + t_g
        out["l2_hit_rate_used"] = h
    return out


def cpu_baseline_and_check(res, torch, target_nnz=80_000_000):
    """Time the serial fp64 oracle on a contiguous block of rows (~target_nnz entries, 10-15 s) and compare GPU rows."""
    from oracle import spmm_csr_oracle  # the only place the benchmark touches the oracle

    p = res.p
    rp = p.rowptr.astype(np.int64)
    start = p.m // 8
    stop = int(np.searchsorted(rp, rp[start] + target_nnz, side="left"))
    stop = max(min(stop, p.m), min(start + 1, p.m))
    rows = np.arange(start, stop, dtype=np.int64)
    sample_nnz = int(rp[stop] - rp[start])
    t0 = time.perf_counter()
    C_ref, _ = spmm_csr_oracle(p.m, p.n, p.rowptr, p.colidx, p.vals, p.B, p.ldb, rows=rows, want_T=False)
    dt = time.perf_counter() - t0
    # the same rows again, split into contiguous chunks over the host cores (each chunk is the same serial loop,
    # so the result is bit-identical); ctypes releases the GIL during the call
    from concurrent.futures import ThreadPoolExecutor
    cores = max(1, min(16, len(os.sched_getaffinity(0))))
    chunks = [c for c in np.array_split(rows, cores) if len(c)]
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as pool:
        parts = list(pool.map(lambda c: spmm_csr_oracle(p.m, p.n, p.rowptr, p.colidx, p.vals, p.B, p.ldb, rows=c,
                                                        want_T=False)[0], chunks))
    dt_par = time.perf_counter() - t0
    same = bool(np.array_equal(np.concatenate(parts), C_ref))
    del parts
    del C_ref
    # parity of the GPU result on EVERY row of the workload (outside the timed parts): the same serial loop, called on
    # contiguous blocks of rows spread over the host cores; each block's C_ref and T are dropped after the comparison
    edges = np.unique(np.concatenate([[0], np.searchsorted(rp, np.linspace(0, rp[-1], 4 * cores + 1)[1:-1]), [p.m]])).astype(np.int64)
    C_host = res.C.cpu().numpy()

    def check_block(b):
        lo, hi = int(edges[b]), int(edges[b + 1])
        ref, T = spmm_csr_oracle(p.m, p.n, p.rowptr, p.colidx, p.vals, p.B, p.ldb, rows=np.arange(lo, hi, dtype=np.int64))
        err = np.abs(C_host[lo:hi].astype(np.float64) - ref)
        bound = 1e-5 * T + 1e-7
        return int(np.count_nonzero(~(err <= bound))), float(np.max(err / bound)) if err.size else 0.0

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as pool:
        checked = list(pool.map(check_block, range(len(edges) - 1)))
    dt_check = time.perf_counter() - t0
    n_bad = sum(c[0] for c in checked)
    worst = max(c[1] for c in checked)
    ok = n_bad == 0
    return {
        "value": 2.0 * sample_nnz * p.n / dt / 1e9,
        "unit": "GFLOP/s",
        "cores": 1,
        "kind": "oracle",
        "sample": f"rows [{start},{stop}) of the same workload: {sample_nnz} nnz, n={p.n}, {dt:.2f} s serial fp64",
        "gpu_matches_oracle_on_every_row": ok,
        "parity": {"rows_checked": int(p.m), "elements_out_of_tolerance": n_bad, "worst_err_over_bound": worst,
                   "tolerance": "|C - C_ref| <= 1e-5 * (|A|.|B|) + 1e-7", "seconds": dt_check},
        "all_cores": {"value": 2.0 * sample_nnz * p.n / dt_par / 1e9, "unit": "GFLOP/s", "cores": len(chunks),
                      "seconds": dt_par, "bit_identical_to_serial": same},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=HEADLINE_CONFIG, help="workload 1..5 of the headline line")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-others", action="store_true", help="skip the short runs of the other four workloads")
    ap.add_argument("--others", type=str, default="1,2,3,4,5", help="which of the other workloads get their short run (comma-separated)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-practical", action="store_true", help="skip the bandwidth probes (practical_peak)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (known traffic) so that a counter run can scale FETCH_SIZE/WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one MI355X); --gpus must be 1. "
              "No multi-GPU path is built.", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2405_16883_amd as sp
    from workloads import CONFIG_NAMES, count_unique_columns, make_config, min_traffic_bytes

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    sp.load_library()
    traffic = load_traffic_table()
    cache = os.environ.get("SCORCH_WORKLOAD_CACHE")

    flush_buf = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0")  # 1 GiB > 256 MB memory-side cache

    def flush():
        flush_buf.add_(1.0)

    practical = None
    if not args.no_practical:
        try:
            practical = measure_practical_peak(torch, flush_buf)
        except Exception as e:  # the probes are benchmark infrastructure: without them the line lacks practical_peak, nothing else
            log(f"[bench] bandwidth probes unavailable ({e}); practical_peak is left out")
    if practical is not None:
        g = practical["row_gather"]
        log(f"[bench] practical peak: stream read {practical['stream_read_2GiB']:.0f} GB/s, copy {practical['copy_1GiB_read_plus_write']:.0f} GB/s, LDS reads {practical['lds_read_b128']:.0f} GB/s; "
            + "; ".join(f"{w} gathers " + "/".join(f"{v:.0f}" for v in g[w].values()) for w in g)
            + " GB/s (table fits one L2 / 2x L2 / 4x L2 / fits the memory-side cache / beyond)")

    def run_config(cfg, steps, warmup, cold_steps):
        t0 = time.perf_counter()
        p = make_config(cfg, seed=args.seed, cache_dir=cache)
        log(f"[bench] cfg {cfg} {CONFIG_NAMES[cfg]}: m={p.m} k={p.k} n={p.n} nnz={p.nnz} generated in {time.perf_counter() - t0:.1f}s")
        bytes_min = min_traffic_bytes(p)
        res = Resident(p, torch, sp)
        wall_ms, ev = time_steps(res, torch, steps, warmup)
        out = summarize(p, wall_ms, ev, bytes_min)
        if cold_steps:
            _, evc = time_steps(res, torch, cold_steps, 1, flush=flush)
            out["cold_event_ms_mean"] = float(np.mean(evc))
            out["cold_frac_hbm"] = bytes_min / (float(np.mean(evc)) * 1e-3) / 1e9 / HBM_PEAK_GBS
        # the plan-free entry point (scorch_spmm_csr) on the same operands, a few calls
        def natural():
            sp.scorch_spmm_csr(p.m, p.k, p.n, res.rowptr, res.colidx, res.vals, res.B, res.C)
        for _ in range(2):
            natural()
        torch.cuda.synchronize()
        nat = []
        for _ in range(5):
            a_, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a_.record()
            natural()
            b_.record()
            nat.append((a_, b_))
        torch.cuda.synchronize()
        out["plan_free_event_ms_mean"] = float(np.mean([x.elapsed_time(y) for x, y in nat]))
        res.step()  # leave the planned result in C
        torch.cuda.synchronize()
        info = res.plan.info()
        out.update({"workload": CONFIG_NAMES[cfg], "m": p.m, "k": p.k, "n": p.n, "nnz": p.nnz,
                    "bytes_min": bytes_min, "plan_ms": res.plan_ms,
                    "plan": {"BN": info.BN, "ALPHA": info.ALPHA, "LW": info.LW, "CH": info.CH, "BCH": info.BCH,
                             "windows": info.n_windows, "short_rows": info.n_short_rows, "wave_rows": info.n_wave_rows,
                             "items": info.n_items, "split_rows": info.n_split_rows,
                             "mode": {0: "gather", 1: "xcd_sliced_gather", 2: "lds_panel"}[info.mode],
                             "hot_columns": info.n_hot_columns, "hot_share": round(float(info.hot_share), 4)}})
        out["mode"] = out["plan"]["mode"]
        tr_ = traffic.get(CONFIG_NAMES[cfg])
        if practical is not None:
            fl = practical_floor(p, bytes_min, count_unique_columns(p), practical, (tr_ or {}).get("l2_hit_rate") if info.mode != 2 else None)
            out["practical_floor"] = fl
            out["frac_of_practical"] = fl["seconds"] / (out["event_ms_mean"] * 1e-3)
            if "seconds_at_measured_l2_hit_rate" in fl:
                out["frac_of_practical_at_measured_l2_hit_rate"] = fl["seconds_at_measured_l2_hit_rate"] / (out["event_ms_mean"] * 1e-3)
        if tr_:
            out["traffic"] = tr_["total_bytes"]
        if info.mode == 2:
            # the panel kernel is bound by plain fp32 multiply-adds out of LDS, not by HBM: price it against the
            # chip's v_fma_f32 rate without packed operations (256 CUs x 64 lanes x 2 flop x 2.4 GHz)
            out["alu_roofline"] = {"bound": "alu", "achieved": out["gflops"] / 1e3, "peak": PLAIN_FMA_TFLOPS,
                                   "unit": "TFLOP/s", "frac": out["gflops"] / 1e3 / PLAIN_FMA_TFLOPS}
        log(f"[bench] cfg {cfg}: {out['event_ms_mean']:.4f} ms/step  {out['gflops']:.0f} GFLOP/s  "
            f"{out['gbs_min_traffic']:.0f} GB/s min-traffic = {100 * out['frac_hbm']:.1f}% of HBM peak  (plan {res.plan_ms:.2f} ms)")
        return res, out

    if args.calibrate_copy:
        src = flush_buf
        dst = torch.empty_like(src)
        dst.copy_(src)  # 1 GiB read + 1 GiB written by one elementwise copy kernel
        torch.cuda.synchronize()
        del dst
    res, head = run_config(args.config, args.steps, args.warmup, cold_steps=5)
    name = CONFIG_NAMES[args.config]
    tr = traffic.get(name)
    roofline = {
        "bound": "hbm",
        "kernel": ("spmm_panel_kernel (+ spmm_pack_b_kernel, same events)" if head["plan"]["mode"] == "lds_panel"
                   else "spmm_fused_kernel (+ spmm_fixup_kernel, same events)"),
        "achieved": head["gbs_min_traffic"],
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": head["frac_hbm"],
        "algorithmic_bytes_per_launch": head["bytes_min"],
        "avg_launch_ms": head["event_ms_mean"],
        "traffic": (tr or {}).get("total_bytes"),
        "traffic_detail": tr,
        "frac_of_peak_on_measured_traffic": ((tr["total_bytes"] / (head["event_ms_mean"] * 1e-3) / 1e9 / HBM_PEAK_GBS)
                                             if tr else None),
        # floor from the rates measured in this run (see practical_floor) over the measured time: above 1 means the
        # kernel beats a reuse-free gather of one row of B per entry, i.e. it already gets reuse out of the caches
        "frac_of_practical": head.get("frac_of_practical"),
        # the same floor with L2 hits priced at the L2-resident gather rate, at the hit rate the committed counter run
        # reports for this kernel: near 1 means the kernel delivers what the cache levels deliver at that hit rate
        "frac_of_practical_at_measured_l2_hit_rate": head.get("frac_of_practical_at_measured_l2_hit_rate"),
        "practical_floor": head.get("practical_floor"),
    }
    cpu = None if args.no_cpu else cpu_baseline_and_check(res, torch)
    if cpu is not None:
        log(f"[bench] cpu oracle: {cpu['value']:.2f} GFLOP/s on 1 core, {cpu['all_cores']['value']:.2f} GFLOP/s on "
            f"{cpu['all_cores']['cores']} cores; GPU matches the oracle on every row: {cpu['gpu_matches_oracle_on_every_row']}")
    del res
    others = {}
    if not args.no_others:
        wanted = {int(x) for x in args.others.split(",") if x.strip()}
        for cfg in (1, 2, 3, 4, 5):
            if cfg == args.config or cfg not in wanted:
                continue
            torch.cuda.empty_cache()
            r, o = run_config(cfg, 50 if cfg != 4 else 20, 5, cold_steps=10 if cfg != 4 else 3)
            if cfg == 1:
                o["graph_replay_ms_per_step"] = time_graph_replay(r, torch, sp)
                log(f"[bench] cfg 1 recorded into a HIP graph (20 steps per replay): {o['graph_replay_ms_per_step'] * 1e3:.2f} us per step")
            if cfg == 2:
                o["sddmm"] = time_sddmm(r, torch, sp, 256)
                log(f"[bench] sddmm on cfg 2 pattern, d=256 (column blocks over the XCDs): {o['sddmm']['event_ms_mean']:.4f} ms  "
                    f"{o['sddmm']['gflops']:.0f} GFLOP/s  {100 * o['sddmm']['frac_hbm']:.1f}% of HBM peak (min-traffic model)")
            if cfg == 3:
                o["sddmm"] = time_sddmm(r, torch, sp, 128)
                log(f"[bench] sddmm on cfg 3 pattern, d=128: {o['sddmm']['event_ms_mean']:.4f} ms  {o['sddmm']['gflops']:.0f} GFLOP/s  "
                    f"{100 * o['sddmm']['frac_hbm']:.1f}% of HBM peak (min-traffic model)")
                o["widenings"] = time_widenings(r, torch, sp)
                w = o["widenings"]
                log(f"[bench] on cfg 3 pattern: spmv {w['spmv']['event_ms_mean'] * 1e3:.1f} us by events, {w['spmv']['graph_replay_ms_per_step'] * 1e3:.1f} us per step in a HIP graph "
                    f"({100 * w['spmv']['frac_hbm_in_a_graph']:.1f}% of HBM peak); "
                    f"spmm+bias+relu fused {w['epilogue']['fused_event_ms_mean'] * 1e3:.1f} us, plain spmm "
                    f"{w['epilogue']['plain_spmm_event_ms_mean'] * 1e3:.1f} us, spmm then elementwise "
                    f"{w['epilogue']['spmm_then_elementwise_event_ms_mean'] * 1e3:.1f} us; GCN layer (width {w['gcn_layer']['width']}) "
                    f"{w['gcn_layer']['event_ms_mean'] * 1e3:.1f} us of which dense product {w['gcn_layer']['dense_product_event_ms_mean'] * 1e3:.1f} us; rowptr from coo "
                    f"{w['formats']['coo_rowptr_event_ms_mean'] * 1e3:.1f} us (ok {w['formats']['coo_matches_rowptr']}), from dcsr "
                    f"{w['formats']['dcsr_rowptr_event_ms_mean'] * 1e3:.1f} us (ok {w['formats']['dcsr_matches_rowptr']})")
            others[CONFIG_NAMES[cfg]] = {k: o[k] for k in ("nnz", "n", "bytes_min", "event_ms_mean", "event_ms_min", "gflops",
                                                           "gbs_min_traffic", "frac_hbm", "cold_event_ms_mean",
                                                           "cold_frac_hbm", "plan_ms", "plan_free_event_ms_mean") + tuple(x for x in ("sddmm", "widenings") if x in o)
                                        + tuple(x for x in ("mode", "traffic", "alu_roofline", "frac_of_practical", "frac_of_practical_at_measured_l2_hit_rate", "practical_floor") if x in o)
                                        + (("graph_replay_ms_per_step",) if "graph_replay_ms_per_step" in o else ())}
            del r

    line = {
        "metric": "SpMM GFLOP/s (2*nnz*n), planned CSR SpMM fp32, 1x MI355X",
        "value": head["gflops"],
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["wall_ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": name, "m": head["m"], "k": head["k"], "n": head["n"], "nnz": head["nnz"],
                   "seed": args.seed, "plan": head["plan"], "plan_ms": head["plan_ms"]},
        "plan_free_ms_per_step": head["plan_free_event_ms_mean"],
        "plan_amortised_in_steps": head["plan_ms"] / head["event_ms_mean"],
        "hbm_gbs_min_traffic": head["gbs_min_traffic"],
        "hbm_frac_of_peak": head["frac_hbm"],
        "cold_cache": {"event_ms_mean": head.get("cold_event_ms_mean"), "frac_hbm": head.get("cold_frac_hbm")},
        "roofline": roofline,
        "practical_peak": practical,
        "cpu_baseline": cpu,
        "other_workloads": others,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
