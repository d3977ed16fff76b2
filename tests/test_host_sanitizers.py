"""The host-side schedule logic (csrc/sched.cpp: state machine, coefficients, divisors, ring weights, threshold
helpers) compiled for the CPU with AddressSanitizer + UndefinedBehaviorSanitizer and driven through seeded random
sequences and its error paths (tests/sched_sanitizer_driver.cpp).  No GPU, no HIP."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host C++ compiler")
def test_sched_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sched_san")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-static-libasan", "-static-libubsan",
           os.path.join(ROOT, "tests", "sched_sanitizer_driver.cpp"), os.path.join(ROOT, "paper_2509_11628_amd", "csrc", "sched.cpp"),
           "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitizer run clean" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
