"""The CPU oracles under AddressSanitizer + UndefinedBehaviorSanitizer (host code only; no GPU involved).

A plain C driver (tests/oracle_sanitize_driver.c) calls every exported function of oracle/akv_oracle.c and
oracle/akw_oracle.c on heap buffers of exactly the documented sizes; this test builds driver + oracles with
-fsanitize=address,undefined -fno-sanitize-recover=all and runs the executable.  Any out-of-bounds access, use of
uninitialised shift counts, signed overflow or misaligned access ends it with a non-zero status and a report."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracles_run_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize_driver")
    build = ["gcc", "-std=c99", "-O1", "-g", "-ffp-contract=off", "-fopenmp", "-fsanitize=address,undefined",
             "-fno-sanitize-recover=all", "-Wall", "-Wextra", "-o", exe,
             os.path.join(ROOT, "tests", "oracle_sanitize_driver.c"), os.path.join(ROOT, "oracle", "akv_oracle.c"),
             os.path.join(ROOT, "oracle", "akw_oracle.c"), "-lm"]
    b = subprocess.run(build, capture_output=True, text=True)
    if b.returncode != 0 and "sanitize" in b.stderr and ("cannot find" in b.stderr or "unrecognized" in b.stderr):
        pytest.skip("the sanitizer runtimes are not installed: " + b.stderr.strip().splitlines()[-1])
    assert b.returncode == 0, b.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "clean" in r.stdout
