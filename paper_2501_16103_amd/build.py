"""Compile the HIP sources into libmoe_sb.so (gfx950 only), in-tree."""
from __future__ import annotations

import os
import re
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libmoe_sb.so")
SRC = os.path.join(HERE, "csrc", "moe_sb.hip")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-FP32 instructions are switched off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


# The GEMM kernels count their global->LDS DMA instructions in vmcnt by hand, and register spills are vector
# memory instructions that count there too: a spill inside a kernel whose waits allow DMAs in flight would let a
# wait pass too early.  Only kernels whose every DMA wait is vmcnt(0) may spill (two-stage rings: the 256 x 256
# tile with 32 slack rows, which sits at the 256-register limit).
SPILL_TOLERANT = ("PipeCfgILi256ELi256ELi64ELi2ELi4ELi2ELb0ELi2ELi32E",)


def check_spills(remarks: str) -> None:
    name = None
    for line in remarks.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            continue
        m = re.search(r"remark:\s+VGPRs Spill: (\d+)", line)
        if m and int(m.group(1)) > 0 and name and "gemm" in name and not any(t in name for t in SPILL_TOLERANT):
            raise RuntimeError(f"{name} spills {m.group(1)} vector registers: its hand-counted vmcnt waits would be wrong")


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-Rpass-analysis=kernel-resource-usage", SRC, "-o", LIB]
    res = subprocess.run(cmd, cwd=HERE, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    check_spills(res.stderr)
    if verbose:
        print(" ".join(cmd))
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
