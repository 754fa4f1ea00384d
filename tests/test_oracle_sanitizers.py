"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a small driver calls every
oracle function on awkward inputs; any out-of-bounds access, leak or undefined operation fails the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "selftest"
    subprocess.run(["gcc", "-std=c11", "-g", "-O1", "-ffp-contract=off", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-static-libasan", "-Wall", "-Wextra",
                    os.path.join(ROOT, "oracle", "selftest.c"), "-o", str(exe), "-lm"], check=True, cwd=os.path.join(ROOT, "oracle"))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stderr[-3000:]
    assert "selftest ok" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
