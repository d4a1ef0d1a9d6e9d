"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only, no GPU code is instrumented):

  * the CPU oracle (oracle/convrot_oracle.c), driven by tests/sanitize/oracle_driver.c on exactly sized heap
    buffers for every group size and both code widths;
  * the host side of the C ABI (csrc/convrot_api.hip: validation, size queries, the static-workspace
    bookkeeping), driven by tests/sanitize/abi_driver.cpp with the kernel launchers replaced by stubs
    (tests/sanitize/launch_stubs.cpp) - every call is one that validation must reject or an empty no-op.

The drivers are stand-alone executables (the sanitizer runtimes are linked in), so nothing is preloaded into
the Python process.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1",
           OMP_NUM_THREADS="4")


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    assert r.returncode == 0, " ".join(cmd) + "\n" + r.stdout + r.stderr
    return r.stdout


def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    run(["gcc", "-O1", "-g", "-fopenmp", "-std=c11", "-Wall", "-Wextra", "-fsanitize=address,undefined",
         "-fno-sanitize-recover=all", "-static-libasan", "-o", exe, os.path.join(SAN, "oracle_driver.c"),
         os.path.join(ROOT, "oracle", "convrot_oracle.c"), "-lm"])
    assert "oracle under sanitizers: ok" in run([exe], env=ENV)


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not installed")
def test_c_abi_host_side_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "abi_san")
    # the sanitizers go to the host pass only; the device pass (the static workspace array) is built as usual
    run(["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
         "-fno-sanitize-recover=all", "-I", os.path.join(ROOT, "include"), "-I",
         os.path.join(ROOT, "paper_2512_03673_amd", "csrc"), "-o", exe, os.path.join(SAN, "abi_driver.cpp"),
         os.path.join(SAN, "launch_stubs.cpp"), os.path.join(ROOT, "paper_2512_03673_amd", "csrc", "convrot_api.hip")])
    # leak detection off here: the HIP runtime the executable links keeps its own allocations until exit
    env = dict(ENV, ASAN_OPTIONS="detect_leaks=0")
    assert "C ABI host side under sanitizers: ok" in run([exe], env=env)
