"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/selftest.c runs every oracle function on
heap buffers of exactly the documented sizes over the edge shapes of the method and re-checks the invariants the paper
fixes; a read or write past an operand, a signed overflow or a misaligned access fails the run.  Host code only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_selftest_is_clean_under_asan_and_ubsan(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_selftest")
    cmd = [gcc, "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-static-libasan", "-Wall", "-Wextra", "-o", exe,
           os.path.join(ROOT, "oracle", "selftest.c"), os.path.join(ROOT, "oracle", "gpusq_oracle.c"), "-lm"]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and ("asan" in build.stderr.lower() or "sanitize" in build.stderr.lower()):
        pytest.skip("this gcc has no sanitizer runtimes: " + build.stderr[-300:])
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert "selftest ok" in run.stdout and "ERROR: AddressSanitizer" not in run.stderr and "runtime error" not in run.stderr
