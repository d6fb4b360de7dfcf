"""Host-side sanitizers over the library's host code (GPU code is never built with sanitizers):
tests/host_check.cpp drives every entry point with made-up device addresses
against stub launchers that check their launch arguments, in a host-only build of csrc/api.hip
with AddressSanitizer and UndefinedBehaviorSanitizer. No GPU is involved."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_15508_amd", "csrc")


def test_host_code_is_clean_under_asan_and_ubsan():
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "host_check")
        subprocess.run([hipcc, "--cuda-host-only", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
                        "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                        "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                        os.path.join(CSRC, "api.hip"), "-x", "hip", os.path.join(ROOT, "tests", "host_check.cpp"), "-o", exe],
                       check=True, capture_output=True, text=True)
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0")   # the HIP runtime keeps its own allocations
        r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
        assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
        assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-2000:]
        assert "host checks done" in r.stdout
