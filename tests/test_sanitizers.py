"""The CPU-side code once under AddressSanitizer and UndefinedBehaviorSanitizer: the oracle (oracle/mesa_ref.c, driven
by tests/san_driver.c over every exported function with exactly sized heap buffers) and the host-side integer helpers
of the product (csrc/host_math.hpp, the program of tests/test_abi_host.py).  Host code only: no GPU code is built or run."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = {**os.environ, "ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "UBSAN_OPTIONS": "print_stacktrace=1:halt_on_error=1",
       "OMP_NUM_THREADS": "2"}
ENV.pop("LD_PRELOAD", None)   # the sanitizer runtime must come first in the list of loaded libraries


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_runs_clean_under_address_and_undefined_behaviour_sanitizers():
    with tempfile.TemporaryDirectory() as d:
        exe = os.path.join(d, "san_oracle")
        subprocess.run(["gcc", "-std=c11", *SAN, "-ffp-contract=off", "-fopenmp", os.path.join(ROOT, "oracle", "mesa_ref.c"),
                        os.path.join(ROOT, "tests", "san_driver.c"), "-o", exe, "-lm"], check=True)
        out = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
        assert out.returncode == 0 and out.stdout.startswith("OK finite"), (out.stdout[-500:], out.stderr[-3000:])
        assert "runtime error" not in out.stderr and "AddressSanitizer" not in out.stderr, out.stderr[-3000:]


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_integer_helpers_run_clean_under_the_sanitizers():
    from tests.test_abi_host import HOST_TEST
    with tempfile.TemporaryDirectory() as d:
        src = os.path.join(d, "t.cpp")
        open(src, "w").write(HOST_TEST)
        exe = os.path.join(d, "t")
        subprocess.run(["g++", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "paper_2111_11124_amd", "csrc"), src, "-o", exe], check=True)
        out = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=600)
        assert out.returncode == 0 and out.stdout.strip() == "OK", (out.stdout[-500:], out.stderr[-3000:])
        assert "runtime error" not in out.stderr, out.stderr[-3000:]
