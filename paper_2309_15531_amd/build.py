"""Builds libadadim.so (HIP, gfx950) in-tree with hipcc: one object per source file, compiled side by
side, then one link.  `build()` compiles every source every time; `build(incremental=True)` (or
`python -m paper_2309_15531_amd.build --incremental`) skips sources whose object is newer than every
file under csrc/ and include/."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libadadim.so")
SOURCES = ["api.hip", "quantize.hip", "hessian.hip", "layer_error.hip", "gemv_ic.hip", "gptq.hip", "probe.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                      # one rounding per operation in the quantizer
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-Wno-inline-asm",                        # the LDS-DMA helper names m0 as clobbered on purpose
]


def _newest_header() -> float:
    t = 0.0
    for d in (CSRC, INCLUDE):
        for f in os.listdir(d):
            if f.endswith(".h"):
                t = max(t, os.path.getmtime(os.path.join(d, f)))
    return t


def build(verbose: bool = True, incremental: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    hdr = _newest_header()

    def compile_one(src: str) -> str:
        s, o = os.path.join(CSRC, src), os.path.join(OBJ, src + ".o")
        if incremental and os.path.exists(o) and os.path.getmtime(o) > max(hdr, os.path.getmtime(s)):
            return o
        cmd = [hipcc, *FLAGS, "-c", s, "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return o

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(incremental="--incremental" in sys.argv[1:])
    sys.exit(0)
