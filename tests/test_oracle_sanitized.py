"""The CPU side under sanitizers: the oracle and a driver that walks it over every shape class,
compiled with -fsanitize=address,undefined (host code; the GPU library is not involved)."""
import os
import shutil
import subprocess

import pytest

from oracle import build_oracle


def test_oracle_is_clean_under_asan_and_ubsan():
    if shutil.which("gcc") is None:
        pytest.skip("gcc not installed")
    try:
        exe = build_oracle.build_sanitized()
    except subprocess.CalledProcessError as e:   # e.g. the sanitizer runtimes are not installed
        pytest.skip(f"cannot build with sanitizers: {e}")
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitize_check: clean" in r.stdout
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr
