"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/selftest.cpp calls every entry
point on small random inputs (graphs with and without self-loops, hub rows, more chunks than vertices, optional
outputs left out); any out-of-bounds access, leak or undefined operation aborts it."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_selftest_under_sanitizers(tmp_path):
    exe = str(tmp_path / "orc_selftest")
    cmd = ["g++", "-O1", "-g", "-fopenmp", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-o", exe, os.path.join(ROOT, "oracle", "selftest.cpp")]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "static-libasan" in built.stderr + built.stdout:
        pytest.skip("no static AddressSanitizer runtime in this toolchain")
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, OMP_NUM_THREADS="2", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    sys.stdout.write(run.stdout)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "oracle selftest: ok" in run.stdout and "runtime error" not in run.stderr
