"""Host logic of the GEMM planning (csrc/streamk.hpp, csrc/layout.hpp), checked by brute-force C++
programs compiled with the host compiler under the address and undefined-behaviour sanitizers:
  * the balanced K split: every workgroup's segments for a range of (tiles per group, K slabs,
    workgroups per group) give exact single coverage, valid slot numbers and load balance;
  * the carving of the `saved` buffer and the two workspaces, and the K partitions the planner
    picks, over a range of shapes and compute-unit counts.
The headers are the ones the kernels and the entry points include."""

import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-g", "-O1", "-std=c++17"]


def _build_and_run(tmp_path, name, min_cases):
    exe = str(tmp_path / name)
    src = os.path.join(ROOT, "tests", "cpp", name + ".cpp")
    subprocess.run(["g++", *SAN, src, "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.startswith("ok "), r.stdout + r.stderr
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr
    assert int(r.stdout.split()[1]) > min_cases


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host C++ compiler")
def test_streamk_partition_bruteforce_under_sanitizers(tmp_path):
    _build_and_run(tmp_path, "streamk_check", 10000)


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host C++ compiler")
def test_buffer_carving_and_k_partitions_under_sanitizers(tmp_path):
    _build_and_run(tmp_path, "layout_check", 500)
