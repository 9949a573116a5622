"""The C oracle rebuilt under AddressSanitizer and UndefinedBehaviorSanitizer (host code only) and run, in a
process of its own, over the cases that touch every one of its buffers: brute-force twin against the two-pass
routine, a row subset, S = 1, argument errors.  A finding of either sanitizer aborts the driver."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-O1", "-g", "-fopenmp",
           "-Wall", "-Wextra", "-o", exe, os.path.join(ROOT, "tests", "csrc", "oracle_sanitized_driver.c"),
           os.path.join(ROOT, "oracle", "attn_oracle.c"), "-lm"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0 and "asan" in res.stderr.lower() and "cannot find" in res.stderr.lower():
        pytest.skip("this gcc has no sanitizer runtime to link")
    assert res.returncode == 0, res.stderr
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="abort_on_error=0:detect_leaks=1",
               UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    if run.returncode != 0 and "does not come first in initial library list" in run.stderr:
        pytest.skip("a preloaded library keeps the sanitizer runtime from starting in this environment")
    assert run.returncode == 0 and "sanitized oracle ok" in run.stdout, run.stdout + run.stderr
