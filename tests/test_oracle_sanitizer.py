"""The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only): a C driver
(oracle/sanitize_check.c) calls every oracle function on small inputs with exactly sized buffers;
any out-of-bounds access, leak or undefined arithmetic makes the run fail."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_address_and_ub_sanitizers(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "sanitize_check")
    cmd = [gcc, "-O1", "-g", "-std=gnu99", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-static-libasan", "-fopenmp", "-Wall", os.path.join(ROOT, "oracle", "sanitize_check.c"), "-o", exe, "-lm"]
    build = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert build.returncode == 0, build.stdout
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout
    assert "sanitize_check: ok" in run.stdout and "runtime error" not in run.stdout and "ERROR: AddressSanitizer" not in run.stdout
