"""GCN layer H' = act(A_hat H W + b) (paper, Section 5.1) through paper_2405_16883_amd.gcn.GcnLayer.

The sparse part is checked to the SpMM tolerance against the fp64 oracle applied to the very dense operand the GPU
kernel was given (the fp32 product H W that torch computed, or H itself); the whole layer is checked against an fp64
numpy evaluation with a tolerance that also covers the fp32 dense product, which is not this library's arithmetic.
"""
import numpy as np
import pytest
import torch

from oracle import spmm_bias_act_oracle, spmm_csr_oracle
from paper_2405_16883_amd.gcn import GcnLayer
from workloads import make_scaled_config

from gpu_util import ATOL, RTOL_T

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")


@pytest.mark.parametrize("n_in,n_out", [(128, 40), (64, 64), (16, 128), (100, 7)])
@pytest.mark.parametrize("relu,with_bias", [(True, True), (False, False)])
def test_gcn_layer_matches_the_oracle(n_in, n_out, relu, with_bias):
    p = make_scaled_config(3, 0.05, seed=11)  # symmetric-normalised power-law graph with self-loops
    rng = np.random.default_rng(n_in * 1000 + n_out)
    H = rng.standard_normal((p.m, n_in)).astype(np.float32)
    W = (rng.standard_normal((n_in, n_out)) / np.sqrt(n_in)).astype(np.float32)
    b = rng.standard_normal(n_out).astype(np.float32) if with_bias else None
    layer = GcnLayer(p.m, torch.from_numpy(p.rowptr).to(DEV), torch.from_numpy(p.colidx).to(DEV),
                     torch.from_numpy(p.vals).to(DEV), p.nnz)
    Hd, Wd = torch.from_numpy(H).to(DEV), torch.from_numpy(W).to(DEV)
    bd = torch.from_numpy(b).to(DEV) if with_bias else None
    out = layer.forward(Hd, Wd, bd, relu=relu).cpu().numpy().astype(np.float64)
    assert layer.aggregates_first(n_in, n_out) == (n_out > n_in)

    if not layer.aggregates_first(n_in, n_out):
        Z = torch.mm(Hd, Wd).cpu().numpy()  # the operand the aggregation kernel saw
        ref, T = spmm_bias_act_oracle(p.m, n_out, p.rowptr, p.colidx, p.vals, Z, b, relu, n_out)
        assert (np.abs(out - ref) <= RTOL_T * T + ATOL).all(), "aggregation + epilogue out of tolerance"
    else:
        Y = torch.empty((p.m, n_in), dtype=torch.float32, device=DEV)
        import paper_2405_16883_amd as sp
        sp.scorch_spmm_csr_planned(layer._plan(n_in), layer.rowptr, layer.colidx, layer.vals, Hd, Y)
        torch.cuda.synchronize()
        ref, T = spmm_csr_oracle(p.m, n_in, p.rowptr, p.colidx, p.vals, H, n_in)
        assert (np.abs(Y.cpu().numpy() - ref) <= RTOL_T * T + ATOL).all(), "aggregation out of tolerance"

    # whole layer in fp64 (either order is the same product)
    AH, _ = spmm_csr_oracle(p.m, n_in, p.rowptr, p.colidx, p.vals, H, n_in)
    full = AH @ W.astype(np.float64)
    if with_bias:
        full = full + b.astype(np.float64)
    if relu:
        full = np.maximum(full, 0.0)
    scale = np.abs(AH) @ np.abs(W.astype(np.float64)) + 1.0
    assert (np.abs(out - full) <= 1e-4 * scale).all(), "layer differs from the fp64 evaluation"
    layer.close()
