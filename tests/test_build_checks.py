"""The build's own checks: what the compiler reports about each kernel is parsed, and a kernel that spills to
scratch memory or misses the occupancy its launch bounds promise fails the build."""
import pytest

from paper_2511_16047_amd import build

REMARKS = """
a.hip:1:1: remark: Function Name: _ZN5amskv12_GLOBAL__N_118attend_bf16_kernelILi64ELi1ELi8ELi64ELi4EEEvPKDF16bPDF16bPcS5_ixNS_8SegTableENS_5ExtKVENS_8CallerIoEfii [-Rpass-analysis=kernel-resource-usage]
a.hip:1:1: remark:     TotalSGPRs: 96 [-Rpass-analysis=kernel-resource-usage]
a.hip:1:1: remark:     VGPRs: 128 [-Rpass-analysis=kernel-resource-usage]
a.hip:1:1: remark:     AGPRs: 0 [-Rpass-analysis=kernel-resource-usage]
a.hip:1:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]
a.hip:1:1: remark:     Dynamic Stack: False [-Rpass-analysis=kernel-resource-usage]
a.hip:1:1: remark:     Occupancy [waves/SIMD]: 4 [-Rpass-analysis=kernel-resource-usage]
a.hip:1:1: remark:     LDS Size [bytes/block]: 65536 [-Rpass-analysis=kernel-resource-usage]
"""


def test_resource_remarks_are_parsed():
    rows = build.kernel_resources(REMARKS)
    assert rows == [{"name": "attend_bf16_kernel<64, 1, 8, 64, 4>", "sgprs": 96, "vgprs": 128, "agprs": 0, "scratch": 0,
                     "occupancy": 4, "lds": 65536}]
    build.check_resources(rows)


@pytest.mark.parametrize("row,word", [
    ({"name": "attend_bf16_kernel<64, 1, 8, 64, 4>", "scratch": 0, "occupancy": 3}, "promise 4"),
    ({"name": "attend_bf16_kernel<128, 1, 4, 32, 3>", "scratch": 12, "occupancy": 3}, "scratch"),
    ({"name": "attend_bf16_small_kernel<64>", "scratch": 0, "occupancy": 3}, "promise 4"),
    ({"name": "compact_kernel", "scratch": 4, "occupancy": 8}, "scratch"),
])
def test_a_spill_or_a_missed_occupancy_fails_the_build(row, word):
    with pytest.raises(build.ResourceError) as e:
        build.check_resources([row])
    assert word in str(e.value)


def test_public_header_is_plain_c():
    """include/amskv.h is the boundary: it must compile by itself as C99 and as C++11 (no torch, no HIP types)."""
    import os
    import subprocess
    header = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "amskv.h")
    for cmd in (["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", header],
                ["g++", "-std=c++11", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c++", header]):
        p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert p.returncode == 0, p.stdout
