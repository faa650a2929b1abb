"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer: a small driver (oracle/sanitize_check.c)
calls every entry point on seeded inputs of many small shapes.  Host code only; nothing here touches a GPU."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_runs_clean_under_sanitizers(tmp_path):
    exe = str(tmp_path / "sanitize_check")
    build = subprocess.run(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                            "-static-libasan", "-static-libubsan",
                            "-ffp-contract=off", "-fopenmp", "-o", exe,
                            os.path.join(ROOT, "oracle", "sanitize_check.c"), os.path.join(ROOT, "oracle", "pq_oracle.c"),
                            "-lm"], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", OMP_NUM_THREADS="2")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "sanitized oracle run: ok" in run.stdout
