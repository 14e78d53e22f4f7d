"""The oracle's C code under AddressSanitizer + UndefinedBehaviorSanitizer (host code only).

oracle/sanitize_check.c calls every oracle entry point on seeded random instances with heap buffers of
exactly the documented sizes; an access past any of them, a leak, or undefined arithmetic aborts it."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_check")
    build = subprocess.run(
        ["gcc", "-O1", "-g", "-std=gnu11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-fno-omit-frame-pointer", "-static-libasan", "-fopenmp", os.path.join(ROOT, "oracle", "metro_oracle.c"),
         os.path.join(ROOT, "oracle", "sanitize_check.c"), "-lm", "-o", exe], capture_output=True, text=True, timeout=300)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", OMP_NUM_THREADS="4")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "sanitize_check: ok" in run.stdout
