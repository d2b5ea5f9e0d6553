"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code; no GPU involved): a
driver calls every exported function on small ragged shapes with exactly sized heap buffers."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not found")
def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    build = subprocess.run(
        ["gcc", "-std=c11", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
         "-fno-sanitize-recover=all", "-static-libasan", "-fopenmp", "-o", exe,
         os.path.join(ROOT, "tests", "native", "oracle_sanitize_main.c"), os.path.join(ROOT, "oracle", "lot_oracle.c"),
         "-lm"], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "oracle sanitize run: ok" in run.stdout
    assert "ERROR" not in run.stderr and "runtime error" not in run.stderr, run.stderr
