"""The host side of the library under AddressSanitizer and UndefinedBehaviorSanitizer.

csrc/kvx_api.hip (configuration checks, arena and scratch layout, per-cache bookkeeping, the packing of
kv_export and kv_import) is compiled for the CPU with g++ against tests/hip_stub/ (a stand-in for the HIP runtime:
host memory, no launches) and driven by tests/hip_stub/host_check.cpp: streams crossing the budget, chunk, batched
and no-allocation calls, every error path, and import -> export -> import -> export round trips in both metadata
formats, both layouts and all code widths.  Any out-of-bounds access, leak or undefined operation fails the run.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
STUB = os.path.join(ROOT, "tests", "hip_stub")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_code_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_check")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-static-libasan", "-I", STUB, "-I", os.path.join(ROOT, "paper_2601_01204_amd", "csrc"), "-x", "c++",
           os.path.join(ROOT, "paper_2601_01204_amd", "csrc", "kvx_api.hip"), os.path.join(STUB, "launch_stubs.cpp"),
           os.path.join(STUB, "host_check.cpp"), "-o", exe, "-lpthread"]
    b = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert b.returncode == 0, b.stderr[-4000:]
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "host checks passed" in r.stdout
