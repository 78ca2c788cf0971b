"""Host logic of the balanced K split (csrc/streamk.hpp): a brute-force C++ checker,
compiled with the host compiler, enumerates every workgroup's segments for a range of
(tiles per group, K slabs, workgroups per group) and verifies exact single coverage, slot
numbering and load balance.  The header is the one the GEMM and reducing kernels include."""

import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host C++ compiler")
def test_streamk_partition_bruteforce(tmp_path):
    exe = str(tmp_path / "streamk_check")
    src = os.path.join(ROOT, "tests", "cpp", "streamk_check.cpp")
    subprocess.run(["g++", "-O2", "-std=c++17", src, "-o", exe], check=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.startswith("ok "), r.stdout
    assert int(r.stdout.split()[1]) > 10000
