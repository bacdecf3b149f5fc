"""Build-time guard (no GPU): the hot kernels must not touch scratch memory.  A spill or a stack object in one of
them costs more than any tuning gains (a lone wave per SIMD cannot hide scratch latency), and it happens silently
when a change makes the register allocator give up."""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2604_17834_amd", "csrc")
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"

HOT = {
    "asp_bcsr_wide.hip": ["bcsr_spmm_wide_kernel"],
    "asp_bcsr.hip": ["bcsr_spmm_kernel"],
    "asp_bcsr_dma.hip": ["bcsr_spmm_dma_kernel"],
    "asp_bcsr_f32.hip": ["bcsr_f32_spmm_kernel"],
    "asp_wcsr.hip": ["wcsr16_spmm_kernel", "wcsr32_spmm_kernel"],
    "asp_wcsr_bf16.hip": ["wcsr_bf16_spmm_kernel"],
}


@pytest.mark.parametrize("source", sorted(HOT))
def test_hot_kernels_use_no_scratch(source):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not found")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        subprocess.check_call([HIPCC, "-O3", "-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                               "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                               "-S", "--cuda-device-only", "-o", out, os.path.join(CSRC, source)],
                              stderr=subprocess.DEVNULL)
        text = open(out).read()
    seen = 0
    for m in re.finditer(r"\.name:\s+(\S+)\n(?:.*\n)*?\s+\.private_segment_fixed_size:\s+(\d+)", text):
        name, scratch = m.group(1), int(m.group(2))
        if any(k in name for k in HOT[source]):
            seen += 1
            assert scratch == 0, "%s uses %d bytes of scratch per lane" % (name, scratch)
    assert seen >= len(HOT[source])
