"""The CPU oracle built with -fsanitize=address,undefined and driven through every entry point on small, awkward
shapes (tests/oracle_sanitize_main.c): an out-of-bounds index, a signed overflow or a misaligned access in the
oracle aborts the run.  CPU only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_runs_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    build = subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined",
                            "-fno-sanitize-recover=all", "-Wall", "-Wextra", "-o", exe,
                            os.path.join(ROOT, "tests", "oracle_sanitize_main.c"),
                            os.path.join(ROOT, "oracle", "wgrad_oracle.c"), "-lm"], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=1", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "oracle sanitize run ok" in run.stdout
