"""Register budget of the headline kernel, checked at compile time (no GPU): the tiled kernels are bound by vector-ALU
issue, and their 2 x 2 variants lose about a fifth of their throughput when they drop from four waves per SIMD to three.
Called routines count against a kernel's registers, so a change far from the hot loops can cost that wave; this test
recompiles the translation unit of the chained bench kernel with the compiler's resource remarks and checks them."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2511_10909_amd", "csrc")


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_headline_kernel_keeps_four_waves_per_simd():
    cmd = ["hipcc", "-c", os.path.join(CSRC, "emulate_tiled_c1v1.hip"), "-o", os.devnull, "--offload-arch=gfx950", "-O3", "-fPIC",
           "-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Rpass-analysis=kernel-resource-usage"]
    out = subprocess.run(cmd, capture_output=True, text=True, timeout=900)
    assert out.returncode == 0, out.stderr[-2000:]
    # template arguments: 32 x 32 block, 2 x 2 per thread, 32 k staged, groups of 8, accumulator added exactly afterwards,
    # no fold, BF16 values: the kernel bench.py reports as "chained"
    name = "emulate_tiled_kernelILi32ELi32ELi2ELi2ELi32ELi8ELi1ELi0ELi1E"
    blocks = [b for b in out.stderr.split("Function Name:")[1:] if name in b.split("\n")[0]]
    assert len(blocks) == 1, "kernel not found in the resource remarks"
    get = lambda key: int(re.search(key + r":\s*(\d+)", blocks[0]).group(1))
    assert get(r"Occupancy \[waves/SIMD\]") >= 4, blocks[0]
    assert get("VGPRs Spill") == 0 and get("VGPRs") <= 128, blocks[0]
