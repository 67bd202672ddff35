"""The fp64 oracle under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only): oracle/sanitize_main.c includes
the oracle's source, gives it heap blocks of exactly the stated sizes, runs ragged layer forward / backward passes
and re-checks a few pins; any out-of-bounds access, use of freed memory, leak, signed overflow or misaligned access
makes the run fail."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = tmp_path / "oracle_sanitized"
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-Wall", "-Wextra", "-o", str(exe),
           os.path.join(ROOT, "oracle", "sanitize_main.c"), "-lm"]
    build = subprocess.run(cmd, capture_output=True, text=True, cwd=os.path.join(ROOT, "oracle"))
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "oracle under sanitizers: ok" in run.stdout
    assert "ERROR: AddressSanitizer" not in run.stderr and "runtime error" not in run.stderr
