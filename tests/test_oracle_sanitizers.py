"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): every entry point once on a
tiny odd-sized layer with exactly-sized buffers, single-threaded and with OpenMP threads."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("openmp", [False, True])
def test_oracle_runs_clean_under_address_and_undefined_sanitizers(tmp_path, openmp):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-Wall", os.path.join(ROOT, "oracle", "r3_oracle.c"), os.path.join(ROOT, "tests", "oracle_sanitize_driver.c"),
           "-lm", "-o", exe] + (["-fopenmp"] if openmp else [])
    subprocess.check_call(cmd)
    # (verify_asan_link_order=0: a library preloaded into every process of this machine may come first)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:verify_asan_link_order=0",
               OMP_NUM_THREADS="3")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, (r.stdout + r.stderr)[-2000:]
    assert r.stdout.startswith("ok "), r.stdout
