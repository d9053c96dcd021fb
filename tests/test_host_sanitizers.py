"""The host-only sources of the library (schedule generator, tuning switches, error text) built with
AddressSanitizer and UndefinedBehaviorSanitizer by the host compiler and driven through the C ABI by
tests/host_sanitizer/driver.cpp.  The GPU sanitizers are not available; kernels are covered by the
parity tests instead."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2405_15362_amd", "csrc")


def test_host_code_under_asan_and_ubsan(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "host_sanitizer_driver")
    srcs = [os.path.join(CSRC, f) for f in ("schedule.cpp", "tuning.cpp", "error.cpp")]
    srcs.append(os.path.join(ROOT, "tests", "host_sanitizer", "driver.cpp"))
    build = subprocess.run([gxx, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                            "-fno-sanitize-recover=all", "-Wall", "-o", exe, *srcs], capture_output=True, text=True)
    if build.returncode != 0 and "sanitize" in build.stderr and "cannot find" in build.stderr:
        pytest.skip("sanitizer runtime not installed")
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    if run.returncode != 0 and "runtime does not come first" in run.stderr:
        pytest.skip("a preloaded library keeps the sanitizer runtime from coming first in this environment")
    assert run.returncode == 0, run.stdout + run.stderr
    assert "passes generated" in run.stdout
