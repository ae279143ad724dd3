"""Host sanitizers (AddressSanitizer + UndefinedBehaviorSanitizer, CPU builds only):
  * the C oracle, compiled into a small driver that runs every exported function on exactly sized
    heap arrays (tests/sanitize/oracle_driver.c);
  * the host side of the C ABI: the library's API translation unit rebuilt with the sanitizers on its
    host code (device code and the other translation units unchanged) and driven through every
    argument check that returns before device work (tests/sanitize/abi_driver.cpp).
Each test builds its program in a temporary directory and requires a clean exit with no sanitizer
report.  No GPU is involved."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1", OMP_NUM_THREADS="2")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    return r.returncode, r.stdout + r.stderr


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    rc, out = _run(["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-o", exe,
                    os.path.join(SAN, "oracle_driver.c"), "-lm"])
    assert rc == 0, out
    rc, out = _run([exe], env=ENV)
    print(out)
    assert rc == 0 and "oracle sanitizer driver: ok" in out, out
    assert "ERROR: AddressSanitizer" not in out and "runtime error" not in out, out


@pytest.mark.slow
def test_abi_argument_checks_under_host_sanitizers(tmp_path):
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not found")
    from paper_2202_13638_amd import build
    build.build()                                    # the other translation units, as the library has them
    objs = [os.path.join(build.BUILD, s.replace(".hip", ".o")) for s in build.SOURCES if s != "bagel_api.hip"]
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer"]
    api_o = str(tmp_path / "bagel_api_san.o")
    rc, out = _run(["hipcc", *build.FLAGS, "-g", *san, "-c", os.path.join(build.CSRC, "bagel_api.hip"), "-o", api_o])
    assert rc == 0, out
    drv_o = str(tmp_path / "abi_driver.o")
    rc, out = _run(["hipcc", "--offload-arch=gfx950", "-std=c++17", "-g", *san, "-I", os.path.join(ROOT, "include"),
                    "-c", os.path.join(SAN, "abi_driver.cpp"), "-o", drv_o])
    assert rc == 0, out
    exe = str(tmp_path / "abi_san")
    rc, out = _run(["hipcc", "--offload-arch=gfx950", "-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined",
                    "-o", exe, drv_o, api_o, *objs])
    assert rc == 0, out
    # the HIP runtime keeps process-lifetime allocations of its own: leak checking is for the oracle driver
    env = dict(ENV, ASAN_OPTIONS=ENV["ASAN_OPTIONS"].replace("detect_leaks=1", "detect_leaks=0"))
    rc, out = _run([exe], env=env)
    print(out)
    assert rc == 0 and "abi sanitizer driver: ok" in out, out
    assert "ERROR: AddressSanitizer" not in out and "runtime error" not in out, out
