"""Host-side checks that need no GPU: the shared library loads and exports what the header declares."""
import ctypes
import os
import re

import pytest

import paper_2405_16883_amd as sp


def declared_functions(repo_root):
    text = open(os.path.join(repo_root, "include", "scorch_spmm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(scorch_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(repo_root):
    if not os.path.exists(sp.LIB_PATH):
        pytest.skip("library not built (run __graft_entry__.build())")
    names = declared_functions(repo_root)
    assert set(names) == set(sp.EXPORTS)
    lib = ctypes.CDLL(sp.LIB_PATH)
    for name in names:
        assert getattr(lib, name) is not None


def test_host_only_calls(repo_root):
    if not os.path.exists(sp.LIB_PATH):
        pytest.skip("library not built")
    lib = sp.load_library()
    assert lib.scorch_status_string(0) == b"ok"
    assert lib.scorch_status_string(-3) == b"workspace too small"
    # workspace bound: host arithmetic only, grows with nnz, rejects nnz >= 2^31
    a = sp.scorch_spmm_plan_workspace_bytes(1000, 1000, 128, 10_000)
    b = sp.scorch_spmm_plan_workspace_bytes(1000, 1000, 128, 10_000_000)
    assert 0 < a < b
    with pytest.raises(sp.ScorchError) as e:
        sp.scorch_spmm_plan_workspace_bytes(10, 10, 4, 2**31)
    assert e.value.status == sp.binding.SCORCH_ERR_UNSUPPORTED
    with pytest.raises(sp.ScorchError) as e:
        sp.scorch_spmm_plan_workspace_bytes(-1, 5, 4, 5)
    assert e.value.status == sp.binding.SCORCH_ERR_INVALID_ARG


def test_binding_refuses_cpu_tensors():
    import torch
    if not os.path.exists(sp.LIB_PATH):
        pytest.skip("library not built")
    z = torch.zeros(3, dtype=torch.int32)
    with pytest.raises(ValueError):
        sp.scorch_spmm_csr(2, 2, 2, z, z, torch.zeros(3), torch.zeros(2, 2), torch.zeros(2, 2))
