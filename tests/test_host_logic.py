"""Host-side logic of the library that needs no GPU: the workgroup -> (column tile, row work) mapping of the
XCD-sliced launches is plain integer arithmetic in a header without HIP dependencies; a small C++ checker
(tests/host/xcd_map_check.cpp) is compiled with the host compiler and run on the CPU."""
import os
import shutil
import subprocess

import pytest


def test_xcd_sliced_workgroup_mapping_covers_every_tile_once(repo_root, tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no host C++ compiler")
    exe = tmp_path / "xcd_map_check"
    src = os.path.join(repo_root, "tests", "host", "xcd_map_check.cpp")
    inc = os.path.join(repo_root, "paper_2405_16883_amd", "csrc")
    subprocess.run([gxx, "-O1", "-std=c++17", "-Wall", "-Werror", "-I" + inc, src, "-o", str(exe)], check=True)
    res = subprocess.run([str(exe)], stdout=subprocess.PIPE, text=True)
    assert res.returncode == 0 and res.stdout.startswith("ok "), res.stdout
    assert int(res.stdout.split()[1]) == 2 * 41 * 10  # every case of the sweep was checked
