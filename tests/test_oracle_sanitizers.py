"""The oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code, CPU only): oracle/sanitize_driver.c
calls every oracle function on ragged, exactly sized heap buffers; any access outside a buffer or undefined
arithmetic inside moa_ref.c aborts the program."""
import os
import subprocess

import pytest


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    import oracle as orc
    try:
        exe = orc.build_sanitize_driver(tmp_path)
    except subprocess.CalledProcessError as e:                       # a toolchain without the sanitizer runtimes
        pytest.skip(f"sanitizer build not available: {e}")
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitize_driver: ok" in r.stdout
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr
