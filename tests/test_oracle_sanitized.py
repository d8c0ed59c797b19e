"""The oracle's C element loops under AddressSanitizer and UBSan (host only).

A small C driver (tests/oracle_sanitizer_driver.c) is linked with
oracle/slowmo_oracle.c, built with -fsanitize=address,undefined, and run on odd
sizes, an empty range and m = 1; any out-of-bounds access or undefined
operation aborts it."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("real,extra", [("double", []), ("float", ["-DORACLE_F32"])])
def test_oracle_loops_are_clean_under_asan_and_ubsan(tmp_path, real, extra):
    exe = str(tmp_path / f"driver_{real}")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-ffp-contract=off",
           f"-DREAL={real}", *extra, "-o", exe,
           os.path.join(ROOT, "tests", "oracle_sanitizer_driver.c"),
           os.path.join(ROOT, "oracle", "slowmo_oracle.c"), "-lm"]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "asan" in (build.stderr + build.stdout).lower():
        pytest.skip("this toolchain has no static AddressSanitizer runtime")
    assert build.returncode == 0, build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0 and run.stdout.strip() == "OK", run.stdout + run.stderr
