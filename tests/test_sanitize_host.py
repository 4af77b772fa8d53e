"""AddressSanitizer + UBSan over the library's host code (no GPU): the scheduling arithmetic
under random use and the argument checks of every GPU entry point, which return before any HIP
call.  The driver is tests/native/sanitize_host.cpp; the library sources are compiled into it
with the host-side sanitizers on (device code is not instrumented)."""
import os
import subprocess

import pytest

from paper_2403_11421_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "native", "sanitize_host.cpp")
OUT_DIR = os.path.join(ROOT, "tests", "native", "_build")


@pytest.mark.skipif(not build.have_compiler(), reason="needs hipcc")
def test_host_code_is_clean_under_asan_and_ubsan():
    os.makedirs(OUT_DIR, exist_ok=True)
    exe = os.path.join(OUT_DIR, "sanitize_host")
    cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-fno-gpu-sanitize",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", build.INCLUDE, "-o", exe] + build.SOURCES + [SRC]
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitize_host: ok" in r.stdout
