"""Runs tests/sanitize_host.py: the library's host code and the C oracle under AddressSanitizer and
UndefinedBehaviorSanitizer, driven by the host tests (no GPU involved)."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_is_clean_under_address_and_ub_sanitizers():
    if os.environ.get("MAMBA_HIP_LIB"):
        pytest.skip("already inside the sanitizer run")
    if not glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"):
        pytest.skip("no shared AddressSanitizer runtime in this image")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "tests", "sanitize_host.py")], capture_output=True, text=True,
                       timeout=900)
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    assert "sanitizer run clean" in r.stdout
