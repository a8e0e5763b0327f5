"""The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only, no GPU):
oracle/tsr_oracle.c is compiled together with a small C driver that calls every routine on ragged
shapes with exactly-sized heap buffers; any out-of-bounds access, leak or undefined operation in
the oracle's loops makes the driver exit non-zero."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_clean_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-fopenmp", "-Wall", "-Wextra", "-o", exe,
           os.path.join(ROOT, "tests", "san", "oracle_sanitize_driver.c"), os.path.join(ROOT, "oracle", "tsr_oracle.c"), "-lm"]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ)
    # the runtime is linked statically, so other preloaded libraries cannot come before it; OpenMP's
    # own thread pool is not freed at exit, which is not a leak of the oracle
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=1:abort_on_error=0"
    env["LSAN_OPTIONS"] = "suppressions=" + os.path.join(ROOT, "tests", "san", "lsan.supp")
    env["OMP_NUM_THREADS"] = "2"
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "sanitize ok" in run.stdout
