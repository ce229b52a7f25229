"""Build the HIP library in-tree: `python -m paper_2105_09377_amd.build`."""

from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libglenside.so")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-inline-asm",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]

# (source, object, extra defines).  The pipelined convolution kernel is instantiated once per
# element type and tile shape, each in its own object so that they compile in parallel.
UNITS = [(src, os.path.splitext(src)[0] + ".o", []) for src in
         ("api.hip", "program.hip", "windows.hip", "gemm.hip", "conv.hip", "conv_smallc.hip", "reduce.hip", "move.hip", "depthwise.hip")]
for _tr, _tag in (("Bf16Traits", "bf16"), ("I8Traits", "i8")):
    for _tile in range(3):
        UNITS.append(("conv3_inst.hip", f"conv3_{_tag}_t{_tile}.o",
                      [f"-DGS_CONV3_TRAITS={_tr}", f"-DGS_CONV3_TILE={_tile}",
                       f"-DGS_CONV3_NAME=launch_conv3_{_tag}_t{_tile}"]))


def _compile(unit) -> str:
    src, obj, defines = unit
    obj = os.path.join(CSRC, obj)
    cmd = ["hipcc", *FLAGS, *defines, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed on " + src)
    noise = "is not a recognized feature for this target"   # printed by the host pass; harmless
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if noise not in l and l.strip())
    if out.strip():
        sys.stderr.write(out + "\n")
    return obj


def build(verbose: bool = True) -> str:
    """Compile every kernel source for gfx950 and link libglenside.so next to this file."""
    workers = min(len(UNITS), max(1, len(os.sched_getaffinity(0))))
    with ThreadPoolExecutor(max_workers=workers) as pool:
        objs = list(pool.map(_compile, UNITS))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
