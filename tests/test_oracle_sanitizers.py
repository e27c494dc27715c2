"""The oracle's C code under AddressSanitizer and UBSan (host only): every routine on small
inputs with exactly sized buffers, all optional parts on.  See oracle/sanitizer_driver.c."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    build = subprocess.run(
        ["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-o", exe, os.path.join(ROOT, "oracle", "sanitizer_driver.c"), "-lm"],
        capture_output=True, text=True)
    if build.returncode != 0 and "sanitize" in build.stderr:
        pytest.skip("this gcc has no sanitizer runtime: " + build.stderr.splitlines()[-1])
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, OMP_NUM_THREADS="3", ASAN_OPTIONS="detect_leaks=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "oracle sanitizer run: ok" in run.stdout
