"""Host-side logic of the library that needs no GPU.  Three pieces of plain integer or text handling live in headers
without HIP dependencies -- the workgroup -> (column tile, row work) mapping of the XCD-sliced launches, the range of
row pointers a key of a coordinate list fills, and the parser of the tuning text -- and small C++ checkers under
tests/host/ are compiled with the host compiler and run on the CPU, once plainly and once under the address and
undefined-behaviour sanitizers.  The C oracles get the same sanitizer pass through a driver that hands them every
operand in a heap block of exactly its size."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import sddmm_csr_oracle, spmm_csr_oracle
from workloads import csr_from_row_lengths

# the sanitizer runtimes are linked statically, so that they need no particular place in the list of loaded libraries
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-static-libasan",
       "-static-libubsan"]
SAN_ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def build_checker(repo_root, tmp_path, name, sanitize, extra=()):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no host C++ compiler")
    exe = tmp_path / (name + ("_san" if sanitize else ""))
    src = os.path.join(repo_root, "tests", "host", name + ".cpp")
    inc = os.path.join(repo_root, "paper_2405_16883_amd", "csrc")
    subprocess.run([gxx, "-O1", "-std=c++17", "-Wall", "-Werror", *(SAN if sanitize else []), "-I" + inc, src, "-o",
                    str(exe), *extra], check=True)
    return str(exe)


def run_checker(exe, sanitize):
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True,
                         env=SAN_ENV if sanitize else None)
    assert res.returncode == 0 and res.stdout.startswith("ok"), res.stdout + res.stderr
    return res.stdout


@pytest.mark.parametrize("sanitize", [False, True])
def test_xcd_sliced_workgroup_mapping_covers_every_tile_once(repo_root, tmp_path, sanitize):
    out = run_checker(build_checker(repo_root, tmp_path, "xcd_map_check", sanitize), sanitize)
    assert int(out.split()[1]) == 2 * 41 * 10  # every case of the sweep was checked


@pytest.mark.parametrize("sanitize", [False, True])
def test_row_pointer_fill_ranges_stay_inside_rowptr(repo_root, tmp_path, sanitize):
    out = run_checker(build_checker(repo_root, tmp_path, "rowptr_keys_check", sanitize), sanitize)
    # sum over m = 0..4 of 2 * sum_{len=0..4} (m + 8)^len key lists
    assert int(out.split()[1]) == sum(2 * sum((m + 8) ** n for n in range(5)) for m in range(5))


@pytest.mark.parametrize("sanitize", [False, True])
def test_tuning_text_parser(repo_root, tmp_path, sanitize):
    run_checker(build_checker(repo_root, tmp_path, "tuning_check", sanitize, extra=("-pthread",)), sanitize)


def sanitized_oracle(repo_root, tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no host C compiler")
    exe = tmp_path / "oracle_san"
    if not exe.exists():
        srcs = [os.path.join(repo_root, "oracle", "spmm_oracle.c"), os.path.join(repo_root, "oracle", "sddmm_oracle.c"),
                os.path.join(repo_root, "tests", "host", "oracle_sanitize_driver.c")]
        subprocess.run([gcc, "-O1", "-std=c99", "-ffp-contract=off", "-Wall", "-Werror", *SAN, *srcs, "-o", str(exe), "-lm"],
                       check=True)
    return str(exe)


def run_sanitized_oracle(exe, tmp_path, m, k, n, ldb, rowptr, colidx, vals, B, rows, X):
    nnz = int(rowptr[-1])
    d = 0 if X is None else X.shape[1]
    path = tmp_path / "problem.txt"
    with open(path, "w") as f:
        f.write(f"{m} {k} {n} {ldb} {nnz} {len(rows)} {d}\n")
        for arr in (rowptr, colidx[:nnz], vals[:nnz], B.reshape(-1), rows, X.reshape(-1) if X is not None else []):
            f.write(" ".join(repr(float(x)) if isinstance(x, (float, np.floating)) else str(int(x)) for x in arr) + "\n")
    res = subprocess.run([exe, str(path)], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=SAN_ENV)
    assert res.returncode == 0, res.stderr[-3000:]
    return np.array(res.stdout.split(), dtype=np.float64)


def test_oracles_under_address_and_undefined_behaviour_sanitizers(repo_root, tmp_path):
    """The hand-worked fixtures and a randomized case (ragged rows, empty rows, ldb > n, a row subset, SDDMM with d = 5)
    run clean under the sanitizers, reproduce the fixtures' printed values, and agree bit for bit with the normal
    build of the same source."""
    from test_oracle_pins import read_fixture

    exe = sanitized_oracle(repo_root, tmp_path)
    for name in ("handworked_3x3.txt", "handworked_signs_4x5.txt"):
        g = read_fixture(name)
        out = run_sanitized_oracle(exe, tmp_path, g["m"], g["k"], g["n"], g["n"], g["rowptr"], g["colidx"], g["vals"],
                                   g["B"], [], None)
        assert np.array_equal(out, np.concatenate([g["C"].reshape(-1), g["T"].reshape(-1)]))
    rng = np.random.default_rng(11)
    lens = np.concatenate([rng.integers(0, 9, size=37), [0, 0, 90, 1]])
    p = csr_from_row_lengths(lens, 23, 7, seed=11, duplicates=True)
    ldb = 9
    B = rng.standard_normal((p.k, ldb)).astype(np.float32)
    X = rng.standard_normal((p.m, 5)).astype(np.float32)
    for rows in ([], [40, 0, 39, 39, 3]):
        out = run_sanitized_oracle(exe, tmp_path, p.m, p.k, p.n, ldb, p.rowptr, p.colidx, p.vals, B, rows, X)
        C, T = spmm_csr_oracle(p.m, p.n, p.rowptr, p.colidx, p.vals, B, ldb, rows=np.array(rows) if rows else None)
        D, TD = sddmm_csr_oracle(p.m, 5, p.rowptr, p.colidx, p.vals, X, B)
        assert np.array_equal(out, np.concatenate([C.reshape(-1), T.reshape(-1), D, TD]))
