"""Compile the HIP library in-tree for gfx950: python -m paper_2206_10620_amd.build"""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libpp_conv.so")

# -packed-fp32-ops: keep the compiler from forming packed FP32 instructions.
# -structurizecfg-skip-uniform-regions: leave the wave-uniform pattern dispatch tree as plain
#   scalar branches (structurising it costs a register copy per accumulator per kernel).
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                "-mllvm", "-structurizecfg-skip-uniform-regions"]
COMMON = ["-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _deps_mtime(src: str, dep: str) -> float:
    """Newest of the source, this script and the project headers the last compile of src read (from its
    depfile); infinity if there is no depfile yet."""
    if not os.path.exists(dep):
        return float("inf")
    names = open(dep).read().replace("\\\n", " ").split()[1:]
    mine = [n for n in names if n.startswith(ROOT)] + [src, os.path.abspath(__file__)]
    return max((os.path.getmtime(n) if os.path.exists(n) else float("inf")) for n in mine)


def _compile(src: str, incremental: bool = False) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    dep = obj + ".d"
    if incremental and os.path.exists(obj) and os.path.getmtime(obj) > _deps_mtime(src, dep):
        return obj
    cmd = ["hipcc"] + COMMON + (DEVICE_FLAGS if src.endswith(".hip") else ["-x", "c++"]) + ["-MD", "-MF", dep, "-c", src, "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"compile failed: {' '.join(cmd)}\n{out}")
    return obj


def build(jobs: int = 8, verbose: bool = False, incremental: bool = False) -> str:
    """Compile every source and link the library.  incremental=True (python -m ... --incremental) keeps
    objects that are newer than their source and every header."""
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.cpp")))
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, incremental), srcs))
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
    subprocess.check_call(cmd)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True, incremental="--incremental" in sys.argv)
    sys.exit(0)
