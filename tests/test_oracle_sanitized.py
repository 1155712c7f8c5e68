"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): oracle/selftest.c walks
every routine over small ragged inputs; any out-of-bounds access, leak, signed overflow or misaligned
access ends the run with a report."""
import os
import shutil
import subprocess
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parents[1]


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_oracle_selftest_under_sanitizers(tmp_path):
    exe = tmp_path / "oracle_selftest"
    # the sanitizer runtime is linked statically: its start-up check of the library order would otherwise
    # object to any library the environment preloads
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-Wall", "-Wextra", "-Werror", str(ROOT / "oracle" / "embedpart_oracle.c"),
           str(ROOT / "oracle" / "selftest.c"), "-o", str(exe), "-lm"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "oracle selftest ok" in run.stdout
