"""The host side of the library (C-ABI argument checks, cache metadata, scheduler) under
AddressSanitizer and UndefinedBehaviorSanitizer: tests/host_sanitize_driver.cpp replaces the
kernel launchers by stubs, is built with the host sources by g++ and run on the CPU."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2511_20426_amd", "csrc")


def test_host_code_is_clean_under_asan_and_ubsan():
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no g++")
    with tempfile.TemporaryDirectory() as d:
        exe = os.path.join(d, "host_sanitize")
        cmd = [cxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
               "-static-libasan", "-static-libubsan", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
               os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"),
               os.path.join(CSRC, "ca_api.cpp"), os.path.join(CSRC, "ca_meta.cpp"), os.path.join(CSRC, "ca_sched.cpp"),
               "-o", exe]
        subprocess.run(cmd, check=True, capture_output=True, text=True)
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
        r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
        assert r.returncode == 0, r.stdout + r.stderr
        assert "host sanitizer driver: ok" in r.stdout
