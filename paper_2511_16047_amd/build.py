"""Compile libamskv.so (HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_2511_16047_amd.build

hipcc cross-compiles without a GPU.  Packed-fp32 instruction selection is switched off for
all device code (see FLAGS).  The build checks what the compiler reports about every kernel
and fails if one of them spills to scratch memory or falls below the number of waves per SIMD
its launch bounds promise: both would be silent performance cliffs (and a spilled asynchronous
load is a correctness hazard in the streaming attention kernel).
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libamskv.so")
OBJ = os.path.join(HERE, "_build")

SOURCES = ["amskv_api.cpp", "cache_kernels.hip", "similarity_kernels.hip", "attend_f32.hip", "attend_bf16.hip", "attend_bf16_small.hip", "density_kernels.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip", "-Wno-inline-asm",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Rpass-analysis=kernel-resource-usage",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]

# Waves per SIMD a kernel must reach (the last template argument of the streaming attention kernel is that
# promise; the coarse-scale and density kernels state theirs in __launch_bounds__).
MIN_OCCUPANCY = [
    (re.compile(r"attend_bf16_kernel<\d+, \d+, \d+, \d+, (\d+)[,>]"), None),     # None: take group 1
    (re.compile(r"attend_density_bf16_kernel<\d+, \d+, \d+, \d+, (\d+)[,>]"), None),
    (re.compile(r"attend_bf16_small_kernel<64>"), 4),
    (re.compile(r"attend_bf16_small_kernel<128>"), 2),
]


class ResourceError(RuntimeError):
    pass


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if p.returncode != 0:
        out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops' is not a recognized feature" not in l)
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return p.stdout


def kernel_resources(compiler_output: str):
    """[{name, sgprs, vgprs, agprs, scratch, occupancy, lds}] from -Rpass-analysis=kernel-resource-usage remarks."""
    rows, cur = [], None
    pat = re.compile(r"remark:\s+(Function Name|TotalSGPRs|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|"
                     r"Occupancy \[waves/SIMD\]|LDS Size \[bytes/block\]): (\S+)")
    key = {"TotalSGPRs": "sgprs", "VGPRs": "vgprs", "AGPRs": "agprs", "ScratchSize [bytes/lane]": "scratch",
           "Occupancy [waves/SIMD]": "occupancy", "LDS Size [bytes/block]": "lds"}
    for line in compiler_output.splitlines():
        m = pat.search(line)
        if not m:
            continue
        k, v = m.groups()
        if k == "Function Name":
            cur = {"name": v}
            rows.append(cur)
        elif cur is not None:
            cur[key[k]] = int(v)
    if rows:
        filt = os.path.join(os.path.dirname(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")), "..", "llvm", "bin", "llvm-cxxfilt")
        filt = filt if os.path.exists(filt) else "c++filt"
        names = subprocess.run([filt] + [r["name"] for r in rows], stdout=subprocess.PIPE, text=True).stdout.splitlines()
        for r, n in zip(rows, names):
            m = re.search(r"N_1\d+([A-Za-z_]\w*?)I((?:L[ib]\d+E)+)E", n)
            if n.startswith("_Z") and m:     # a type this c++filt does not know (__bf16): integer template arguments by hand
                n = "%s<%s>" % (m.group(1), ", ".join(re.findall(r"L[ib](\d+)E", m.group(2))))
            n = n.replace("(anonymous namespace)::", "").replace("void ", "").replace("amskv::", "")
            r["name"] = n.split("(")[0]
    return rows


def check_resources(rows):
    problems = []
    for r in rows:
        if r.get("scratch", 0) != 0:
            problems.append("%s spills %d bytes per lane to scratch memory" % (r["name"], r["scratch"]))
        for pat, want in MIN_OCCUPANCY:
            m = pat.search(r["name"])
            if m:
                need = int(m.group(1)) if want is None else want
                if r.get("occupancy", 0) < need:
                    problems.append("%s reaches %d waves per SIMD, its launch bounds promise %d"
                                    % (r["name"], r.get("occupancy", 0), need))
    if problems:
        raise ResourceError("kernel resource check failed:\n  " + "\n  ".join(problems))


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    objs = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in SOURCES]

    def one(pair):
        src, obj = pair
        return _run([hipcc] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj])

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        outs = list(ex.map(one, zip(SOURCES, objs)))
    rows = [r for o in outs for r in kernel_resources(o)]
    if verbose:
        for r in rows:
            print("%-64s vgpr %3d agpr %3d sgpr %3d scratch %3d lds %6d occupancy %d" % (
                r["name"][-64:], r.get("vgprs", 0), r.get("agprs", 0), r.get("sgprs", 0), r.get("scratch", 0),
                r.get("lds", 0), r.get("occupancy", 0)))
    check_resources(rows)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
    sys.exit(0)
