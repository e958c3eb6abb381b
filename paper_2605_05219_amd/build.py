"""Builds the HIP library in-tree for gfx950 (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libgdn_resume.so")
LIB_PHASES = os.path.join(PKG, "libgdn_resume_phases.so")   # profiling build: the fused kernel leaves cycle stamps
SOURCES = ["gdn_resume.hip", "gdn_layer.hip", "gdn_linear.hip", "attn_resume.hip", "gdn_plan.cpp", "ckpt_place.cpp"]


def build_library(verbose: bool = False, phase_stamps: bool = False) -> str:
    lib = LIB_PHASES if phase_stamps else LIB
    cmd = ["hipcc", "-O3", "--offload-arch=gfx950", "-std=c++17", "-shared", "-fPIC",
           # packed fp32 instructions are switched off for all device code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    if phase_stamps:
        cmd.append("-DGDN_PHASE_STAMPS")
    cmd += [os.path.join(CSRC, s) for s in SOURCES] + ["-o", lib]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building " + os.path.basename(lib))
    return lib


if __name__ == "__main__":
    import sys
    print(build_library(verbose=True, phase_stamps="--phase-stamps" in sys.argv[1:]))
