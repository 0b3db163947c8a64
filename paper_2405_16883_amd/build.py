"""Builds libscorch_spmm.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
OBJ_DIR = os.path.join(PKG_DIR, "_build")
LIB_PATH = os.path.join(PKG_DIR, "libscorch_spmm.so")
SOURCES = ["spmm_api.hip", "spmm_plan.hip", "spmm_exec.hip", "spmm_panel.hip", "sddmm_exec.hip", "spmm_static.hip"]
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # no packed-fp32 VALU forms: keep fp32 multiply-adds as plain v_fma_f32
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build_library(verbose: bool = False) -> str:
    """Compiles every source (in parallel) and links the shared library; always rebuilds."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        hipcc = "hipcc"
    os.makedirs(OBJ_DIR, exist_ok=True)
    inc = ["-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
    objs = [os.path.join(OBJ_DIR, s.replace(".hip", f".{os.getpid()}.o")) for s in SOURCES]
    jobs = min(len(SOURCES), max(1, min(8, os.cpu_count() or 1)))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        list(pool.map(lambda so: _run([hipcc, *HIPCC_FLAGS, *inc, "-c", os.path.join(CSRC, so[0]), "-o", so[1]], verbose),
                      zip(SOURCES, objs)))
    tmp = LIB_PATH + f".tmp{os.getpid()}"
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp], verbose)
    os.replace(tmp, LIB_PATH)
    for o in objs:
        os.remove(o)
    return LIB_PATH


PROBES_LIB_PATH = os.path.join(PKG_DIR, "libscorch_probes.so")


def build_probes(verbose: bool = False) -> str:
    """Builds the benchmark's bandwidth probes into a library of their own (the product library never sees them)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        hipcc = "hipcc"
    tmp = PROBES_LIB_PATH + f".tmp{os.getpid()}"
    _run([hipcc, *HIPCC_FLAGS, "-shared", os.path.join(CSRC, "probes", "bandwidth_probes.hip"), "-o", tmp], verbose)
    os.replace(tmp, PROBES_LIB_PATH)
    return PROBES_LIB_PATH


if __name__ == "__main__":
    print(build_probes(verbose="-v" in sys.argv))
    print(build_library(verbose="-v" in sys.argv))
