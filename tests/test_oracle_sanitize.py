"""Host-side sanitizers over the oracle: the C driver tests/oracle_sanitize_check.c calls every oracle
function (ragged, empty, padded and error cases) in a build with AddressSanitizer and
UndefinedBehaviorSanitizer. GPU code is never built with sanitizers."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_and_ubsan():
    src = [os.path.join(ROOT, "tests", "oracle_sanitize_check.c"), os.path.join(ROOT, "oracle", "sts_oracle.c")]
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "oracle_san")
        subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined",
                        "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-static-libasan",
                        "-I", os.path.join(ROOT, "oracle"), "-o", exe, *src,
                        "-lm"],
                       check=True)
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", OMP_NUM_THREADS="4")
        r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
        assert r.returncode == 0, r.stdout + r.stderr
        assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr
