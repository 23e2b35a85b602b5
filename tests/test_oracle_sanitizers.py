"""The oracle's C code (model, simulator, offline-pruning reference) under AddressSanitizer and
UndefinedBehaviorSanitizer, host side only: tests/c_client/oracle_sanitize.c calls every entry
point on small inputs, at the edges of its index ranges too, and cross-checks what they return."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    build = subprocess.run(
        ["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
         os.path.join(ROOT, "tests", "c_client", "oracle_sanitize.c"), os.path.join(ROOT, "oracle", "offline.c"),
         "-lm", "-o", exe], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    # (a preloaded library may come before the sanitizer runtime in the link order: that is not an error here)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert "oracle under sanitizers: ok" in run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr
