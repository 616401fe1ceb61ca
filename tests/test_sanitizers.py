"""The CPU code under AddressSanitizer and UndefinedBehaviorSanitizer: the oracle (plain C) and the
host side of the library (rsdgc_plan.cpp: plan construction, queries, argument checks) are compiled
with -fsanitize=address,undefined together with a small driver (tests/sanitize/driver.cpp) that
calls every oracle entry point and the plan entry points on small seeded inputs -- ragged shapes,
every neighbourhood side, keep ratios 0 and 1 -- and checks a few invariants on the way.  The
sanitizers abort on the first finding, so a clean exit is the assertion.  No GPU, no HIP."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None or shutil.which("gcc") is None, reason="no host compiler")
def test_oracle_and_host_plan_code_run_clean_under_asan_and_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    oracle_o = tmp_path / "oracle.o"
    subprocess.check_call(["gcc", "-std=c99", "-ffp-contract=off", "-Wall", "-Wextra", *san, "-c",
                           os.path.join(ROOT, "oracle", "rsdgc_oracle.c"), "-o", str(oracle_o)])
    exe = tmp_path / "sanitized"
    subprocess.check_call(["g++", "-std=c++17", "-Wall", *san, "-static-libasan",
                           os.path.join(ROOT, "tests", "sanitize", "driver.cpp"),
                           os.path.join(ROOT, "paper_2312_17530_amd", "csrc", "rsdgc_plan.cpp"),
                           str(oracle_o), "-o", str(exe), "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    proc = subprocess.run([str(exe)], env=env, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=300)
    assert proc.returncode == 0, proc.stdout + proc.stderr
    assert "sanitized run ok" in proc.stdout
