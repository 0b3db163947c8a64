"""The execution entry points neither wait nor allocate, so they can be recorded into a HIP graph.

Each replay is checked against the eager result, with eager work and synchronisations between replays.
"""
import numpy as np
import pytest
import torch

import paper_2405_16883_amd as sp
from workloads import make_scaled_config

from gpu_util import DeviceProblem, check_against_oracle

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg,scale,tune", [(1, 1.0, None), (3, 0.08, None),
                                            (5, 0.06, "sliced=1,pack=1,ch=64,bch=128"),  # pack pre-pass + fix-up launch in the graph
                                            (5, 0.06, "panel=1"), (5, 0.06, "panel=2")])  # copy of B + panel kernel in the graph
def test_planned_spmm_and_sddmm_replay_in_a_graph(cfg, scale, tune, monkeypatch):
    if tune:
        monkeypatch.setenv("SCORCH_SPMM_TUNE", tune)
    p = make_scaled_config(cfg, scale, seed=4)
    d = DeviceProblem(p)
    plan = d.make_plan()
    eager = d.run_planned(plan).copy()
    check_against_oracle(p, eager, d.ldc, label="eager")
    dd = min(p.n, 128)
    X = torch.randn((p.m, dd), device=d.dev)
    Yt = torch.randn((p.k, dd), device=d.dev)
    out = torch.empty(max(p.nnz, 1), device=d.dev)
    sp.scorch_sddmm_csr_planned(plan, dd, d.rowptr, d.colidx, d.vals, X, Yt, out)
    torch.cuda.synchronize()
    eager_sddmm = out.cpu().numpy().copy()

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            sp.scorch_spmm_csr_planned(plan, d.rowptr, d.colidx, d.vals, d._B_arg(), d._C_arg(), stream=side)
            sp.scorch_sddmm_csr_planned(plan, dd, d.rowptr, d.colidx, d.vals, X, Yt, out, stream=side)
    torch.cuda.synchronize()
    for replay in range(4):
        d.Cfull.fill_(-3.0)  # eager work between replays
        out.fill_(-3.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(d.Cfull.cpu().numpy(), eager), f"SpMM replay {replay} differs from the eager result"
        assert np.array_equal(out.cpu().numpy(), eager_sddmm), f"SDDMM replay {replay} differs from the eager result"
    plan.destroy()
