"""The library from a plain C program: tests/c_abi/abi_check.c includes include/amskv.h and the HIP runtime API and
nothing else (no torch, no Python, no C++), allocates with hipMalloc and checks amskv_append_scale / amskv_attend on
fp32 and bf16 caches against Eq. 2 written out in double precision.  The CPU test compiles and links it against the
built library (the header is C, every symbol resolves); the GPU test runs it as a child process.

Bar: exit status 0, i.e. max-abs 1e-4 (fp32) / 2e-2 (bf16) on every output and the kept sets listed by hand.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2511_16047_amd")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def _build(exe):
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    assert os.path.exists(os.path.join(PKG, "libamskv.so")), "libamskv.so is not built (python -m paper_2511_16047_amd.build)"
    cmd = ["gcc", "-std=c11", "-O2", "-Wall", "-Wextra", "-Werror", "-D__HIP_PLATFORM_AMD__", "-isystem", os.path.join(ROCM, "include"),
           "-I" + os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "c_abi", "abi_check.c"), "-o", exe,
           "-L" + PKG, "-lamskv", "-L" + os.path.join(ROCM, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath," + PKG, "-Wl,-rpath," + os.path.join(ROCM, "lib")]
    b = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert b.returncode == 0, b.stdout[-4000:]


def test_c_program_compiles_and_links(tmp_path):
    _build(str(tmp_path / "abi_check"))


@pytest.mark.gpu
def test_c_program_runs(tmp_path):
    exe = str(tmp_path / "abi_check")
    _build(exe)      # a one-second host compile of a C file; the library itself was built beforehand
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    print(r.stdout)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "abi_check: ok" in r.stdout
