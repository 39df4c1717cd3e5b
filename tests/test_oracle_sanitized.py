"""The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer: a C driver
(oracle/sanitize_check.c) calls every entry point on exactly sized buffers; any
out-of-bounds access or undefined index arithmetic aborts the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan",       # runtime linked in: no ordering demands on preloaded libraries
           "-o", exe, os.path.join(ROOT, "oracle", "rib_oracle.c"),
           os.path.join(ROOT, "oracle", "sanitize_check.c"), "-lm"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "asan" in built.stderr.lower():
        pytest.skip("the sanitizer runtime is not installed: " + built.stderr.strip().splitlines()[-1])
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", OMP_NUM_THREADS="4")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.strip() == "ok"
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr
