"""The host layer of the library (csrc/amskv_api.cpp: policy -> kept set, slot planning, Algorithms 1 and 2 on
token lists, status codes) built for the CPU with AddressSanitizer and UndefinedBehaviorSanitizer and walked by
tests/host_sanitize/driver.cpp over plan-only caches.  No GPU, no HIP runtime: the kernel launchers are stubs."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host compiler")
def test_host_layer_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_2511_16047_amd", "csrc"),
           os.path.join(ROOT, "paper_2511_16047_amd", "csrc", "amskv_api.cpp"),
           os.path.join(ROOT, "tests", "host_sanitize", "driver.cpp"), "-o", exe]
    b = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert b.returncode == 0, b.stdout[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "0 check(s) failed" in r.stdout
