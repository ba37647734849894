"""The host-side C++ (planner, chunk scheduler, K/V block manager) under AddressSanitizer and
UndefinedBehaviorSanitizer: tests/host_fuzz.cpp is built with the host compiler (no HIP, no GPU) and run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2412_18106_amd", "csrc")


def test_planner_scheduler_and_block_manager_fuzz_under_asan_and_ubsan(tmp_path):
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path / "host_fuzz")
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer", "-static-libasan", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(ROOT, "tests", "host_fuzz.cpp"), os.path.join(CSRC, "plan.cpp"), os.path.join(CSRC, "serving.cpp"),
           "-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True)
    assert built.returncode == 0, built.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0 and "host_fuzz: ok" in run.stdout, (run.stdout[-2000:], run.stderr[-4000:])
