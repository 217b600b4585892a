"""Compile the HIP sources into libmoe_sb.so (gfx950 only), in-tree."""
from __future__ import annotations

import os
import re
import shutil
import subprocess
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libmoe_sb.so")
SRC = os.path.join(HERE, "csrc", "moe_sb.hip")
# measurement kernels, kept out of the product library
PROBE_LIB = os.path.join(HERE, "libmoe_probe.so")
PROBE_SRC = os.path.join(HERE, "csrc", "moe_probe.hip")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-FP32 instructions are switched off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # The k loops are unrolled completely by pragma; at the default size limit for pragma-unrolled loops the largest
    # copies sit at the edge, and a loop left rolled indexes the accumulators dynamically, which puts them in memory.
    "-mllvm", "-pragma-unroll-threshold=100000",
]


# A register spill inside a k loop is a vector memory instruction among the hand-counted global->LDS DMAs: the
# compiler waits for its reload with vmcnt(0), which drains the whole DMA ring every iteration (measured: a
# third of the throughput gone).  The build therefore reads the device assembly and refuses a GEMM kernel that
# has a scratch access inside a loop that also holds MFMAs.  (Spills outside the loops only cost their own time;
# they cannot let a DMA wait pass early: loads retire in order and extra entries in vmcnt make a wait stricter.)
def check_no_spill_in_k_loops(asm_text: str) -> None:
    # accumulators or fragments that were not promoted to registers show up as a large private segment
    for m in re.finditer(r"\.name:\s+(\S+)\n(?:.*\n)*?\s+\.private_segment_fixed_size:\s+(\d+)", asm_text):
        if "gemm" in m.group(1) and int(m.group(2)) > 256:
            raise RuntimeError(f"{m.group(1)}: {m.group(2)} bytes of private memory per lane (an array left in memory?)")
    for m in re.finditer(r"^(_ZN3moe\S*gemm\S*):\s*(?:;.*)?$", asm_text, re.M):
        name = m.group(1)
        end = asm_text.find(".Lfunc_end", m.end())
        lines = asm_text[m.end():end].splitlines()
        label_at = {ln.split(":")[0]: k for k, ln in enumerate(lines) if ln.startswith(".LBB")}
        loops = []   # (first line, last line) of every backward branch's span

        def exits(k):   # the block at line k does nothing but end the program (an early-placed exit, not a loop head)
            for ln in lines[k + 1:]:
                ln = ln.strip()
                if ln and not ln.startswith(";"):
                    return ln.startswith("s_endpgm")
            return False

        for k, ln in enumerate(lines):
            b = re.search(r"s_cbranch\w*\s+(\.LBB\d+_\d+)", ln)
            if b and label_at.get(b.group(1), len(lines)) < k and not exits(label_at[b.group(1)]):
                loops.append((label_at[b.group(1)], k))
        def mfmas(lo, hi):
            return sum("v_mfma" in lines[x] for x in range(lo, hi + 1))

        for k, ln in enumerate(lines):
            if "scratch_" not in ln:
                continue
            around = [lp for lp in loops if lp[0] <= k <= lp[1]]
            if not around:
                continue
            lo, hi = min(around, key=lambda lp: lp[1] - lp[0])          # the innermost loop around the access
            inner = [lp for lp in loops if lo <= lp[0] and lp[1] <= hi and lp != (lo, hi)]
            if any(mfmas(a, b) >= 16 for a, b in inner):
                # a loop over tiles (resident kernels) with the k loops inside it: a reload between two tiles costs
                # its own time only -- unless it sits in the middle of a straight run of MFMAs (the unrolled last
                # iterations of a tile, which still have DMAs in flight)
                if mfmas(max(lo, k - 40), k) >= 8 and mfmas(k, min(hi, k + 40)) >= 8:
                    raise RuntimeError(f"{name}: register spill among the MFMAs of a tile's last iterations")
                continue
            own = sum("v_mfma" in lines[x] for x in range(lo, hi + 1) if not any(a <= x <= b for a, b in inner))
            if own >= 16:
                raise RuntimeError(f"{name}: register spill inside a k loop (it would drain the DMA ring every iteration)")


def _compile(src: str, lib: str, check_spills: bool, verbose: bool) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, os.path.basename(lib))
        cmd = [hipcc] + HIPCC_FLAGS + ["-save-temps=obj", src, "-o", out]
        res = subprocess.run(cmd, cwd=tmp, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
        if check_spills:
            asm = [f for f in os.listdir(tmp) if f.endswith(".s") and "amdgcn" in f]
            if not asm:
                raise RuntimeError("no device assembly found next to the built library")
            with open(os.path.join(tmp, asm[0])) as f:
                check_no_spill_in_k_loops(f.read())
        shutil.copyfile(out, lib)
        os.chmod(lib, 0o755)
    if verbose:
        print(" ".join(cmd))
    return lib


def build_library(verbose: bool = False) -> str:
    """libmoe_sb.so: the product library."""
    return _compile(SRC, LIB, True, verbose)


def build_probe_library(verbose: bool = False) -> str:
    """libmoe_probe.so: the measurement kernels (bench.py --mfma-probe and two tests load it)."""
    return _compile(PROBE_SRC, PROBE_LIB, False, verbose)


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_probe_library(verbose=True))
