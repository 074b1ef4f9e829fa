"""The oracle's C code under the undefined-behaviour sanitizer: the pin tests are run once more, in a child process,
against a build of the same sources with -fsanitize=undefined (signed overflow, shifts, strict array bounds, float to
integer casts, misaligned and null pointers), every finding fatal.  A pin that only passes because of an out-of-range
shift or an overflowing index would be no pin.  CPU only; the HIP path is not involved."""
import os
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRCS = [os.path.join(ROOT, "oracle", n) for n in ("moe_oracle.c", "moe_oracle_fp8.c")]
PINS = ["test_oracle_router.py", "test_oracle_permute.py", "test_oracle_layer.py", "test_oracle_fp8.py",
        "test_oracle_backward.py", "test_oracle_permute_variants.py", "test_oracle_sort_chunks.py"]


def test_pins_pass_on_a_sanitized_build_of_the_oracle():
    with tempfile.TemporaryDirectory() as tmp:
        lib = os.path.join(tmp, "libmoe_oracle_ubsan.so")
        subprocess.run(["gcc", "-O1", "-g", "-fopenmp", "-shared", "-fPIC",
                        "-fsanitize=undefined,bounds-strict,float-cast-overflow", "-fno-sanitize-recover=all",
                        "-o", lib, *SRCS, "-lm"], check=True)
        env = dict(os.environ, MOE_ORACLE_LIB=lib, UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
        r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                            *[os.path.join(ROOT, "tests", p) for p in PINS]],
                           cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
        out = r.stdout + r.stderr
        assert "runtime error" not in out, out[-3000:]
        assert r.returncode == 0, out[-3000:]
