"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): oracle/sanitize_check.c
calls every entry point on small dense and CSR problems; any report fails the build's run."""
import os
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("openmp", [False, True], ids=["plain", "openmp"])
def test_oracle_is_clean_under_asan_and_ubsan(openmp):
    src = [os.path.join(ROOT, "oracle", "ssn_oracle.c"), os.path.join(ROOT, "oracle", "sanitize_check.c")]
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "sanitize_check")
        cmd = ["gcc", "-O1", "-g", "-std=c99", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
               "-fno-omit-frame-pointer"] + (["-fopenmp"] if openmp else []) + ["-o", exe] + src + ["-lm"]
        subprocess.check_call(cmd)
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", OMP_NUM_THREADS="3")
        out = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
        assert out.returncode == 0, out.stderr[-3000:]
        assert "sanitize_check ok" in out.stdout
        assert "ERROR" not in out.stderr and "runtime error" not in out.stderr, out.stderr[-3000:]
