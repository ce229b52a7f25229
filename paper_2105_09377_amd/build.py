"""Build the HIP library in-tree: `python -m paper_2105_09377_amd.build`."""

from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libglenside.so")
SOURCES = ["api.hip", "windows.hip", "gemm.hip", "conv.hip", "reduce.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed on " + src)
    noise = "is not a recognized feature for this target"   # the host pass does not know the packed-fp32 feature; harmless
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if noise not in l and l.strip())
    if out.strip():
        sys.stderr.write(out + "\n")
    return obj


def build(verbose: bool = True) -> str:
    """Compile every kernel source for gfx950 and link libglenside.so next to this file."""
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
        objs = list(pool.map(_compile, SOURCES))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
