"""Builds liblmk_gs.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2503_21364_amd.build

Every translation unit is compiled with packed-FP32 instruction selection
switched off.  preprocess.hip, binsort.hip and api.hip additionally run with
floating-point contraction off and correctly rounded divide/sqrt, because they
hold the arithmetic that decides integers (depth bits, tile rectangles, culls,
the tile intersection test).
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "liblmk_gs.so")
OBJDIR = os.path.join(HERE, "_build")

ARCH = "gfx950"
COMMON = ["-O3", "-std=c++17", "-fPIC", f"--offload-arch={ARCH}", "-I", INCLUDE, "-I", CSRC,
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wall", "-Wno-unused-command-line-argument"]
EXACT = ["-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt"]
UNITS = {
    "api.hip": EXACT,
    "preprocess.hip": EXACT,
    "binsort.hip": EXACT,       # the tile intersection test of binning rule 1 decides integers too
    "render.hip": [],
    "render_bwd.hip": [],       # same options as render.hip: pass 1 repeats its arithmetic
    "preprocess_bwd.hip": [],
    "anchor_decode.hip": [],
    "index.hip": EXACT,         # host code: the voxel of a primitive is decided by one fp32 division
}


def hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the HIP library cannot be built")


def build(verbose: bool = False) -> str:
    cc = hipcc()
    os.makedirs(OBJDIR, exist_ok=True)
    objs = []
    for unit, extra in UNITS.items():
        obj = os.path.join(OBJDIR, unit.replace(".hip", ".o"))
        cmd = [cc, *COMMON, *extra, "-c", os.path.join(CSRC, unit), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        objs.append(obj)
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [cc, "-shared", "-fPIC", f"--offload-arch={ARCH}", "-o", tmp, *objs,
           "-Wl,-rpath,/opt/rocm/lib", "-Wl,--no-undefined"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
