"""The host-side planner under AddressSanitizer and UndefinedBehaviorSanitizer on the CPU:
random layer tables, worker counts up to 2^20, every radix and order, with the planner's
invariants checked along the way (tests/host/sanitize_planner.cpp)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_planner_under_asan_and_ubsan(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = tmp_path / "sanitize_planner"
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-Wall", "-Wextra", "-Werror",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2006_02924_amd", "csrc"),
           os.path.join(ROOT, "tests", "host", "sanitize_planner.cpp"),
           os.path.join(ROOT, "paper_2006_02924_amd", "csrc", "adasum_plan.cpp"), "-o", str(exe)]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([str(exe), "300"], env=env, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert "planner ok" in res.stdout
