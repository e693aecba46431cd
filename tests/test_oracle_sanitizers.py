"""The C oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only): oracle/sanitize_check.c calls every
entry point on small ragged shapes in buffers of exact size; any report aborts the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    exe = tmp_path / "sanitize_check"
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-fno-omit-frame-pointer", "-Wall", "-o", str(exe), os.path.join(ROOT, "oracle", "antkv_oracle.c"),
           os.path.join(ROOT, "oracle", "sanitize_check.c"), "-lm"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", OMP_NUM_THREADS="4")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "sanitize_check: ok" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]
