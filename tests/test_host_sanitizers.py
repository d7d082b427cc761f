"""The library's host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only, no GPU needed):
csrc/host_check_driver.cpp calls the entry points with device "pointers" that are never dereferenced -- bad arguments,
well-formed single calls, whole steps under every schedule and regime (their checks-only pass walks the workspace carving
and launch planning of every stage) -- and runs the gzip pass of the first message for real."""
import os
import subprocess
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent


def _build_module():
    import importlib.util
    spec = importlib.util.spec_from_file_location("moa_build", ROOT / "paper_2410_03804_amd" / "build.py")
    mod = importlib.util.module_from_spec(spec)
    sys.modules["moa_build"] = mod
    spec.loader.exec_module(mod)
    return mod


def test_host_code_runs_clean_under_asan_and_ubsan(tmp_path):
    build = _build_module()
    try:
        exe = build.build_host_check_driver(tmp_path)
    except (RuntimeError, subprocess.CalledProcessError, OSError) as e:       # a toolchain without the sanitizer runtimes
        pytest.skip(f"sanitizer build not available: {e}")
    # leak detection is off: the HIP runtime keeps its own allocations for the life of the process
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host_check_driver: ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr
