"""The library's host-side planning code (tiling of the tensor list, update
order of a mixing step) under AddressSanitizer and UBSan, host only: the
driver tests/plan_sanitizer_driver.cpp is built with csrc/slowmo_plan.cpp (no
HIP in either) and run on random tensor lists and in-neighbour maps."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1910_00643_amd", "csrc")


def test_planning_code_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "plan_driver")
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-ffp-contract=off", "-I", CSRC,
           "-o", exe, os.path.join(ROOT, "tests", "plan_sanitizer_driver.cpp"),
           os.path.join(CSRC, "slowmo_plan.cpp")]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "asan" in (build.stderr + build.stdout).lower():
        pytest.skip("this toolchain has no static AddressSanitizer runtime")
    assert build.returncode == 0, build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0 and run.stdout.strip() == "OK", run.stdout + run.stderr
