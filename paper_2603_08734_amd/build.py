"""Build the HIP library in-tree (``librsh.so`` next to this file) for gfx950."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librsh.so")
SOURCES = ["kernels.hip", "api.cpp", "planner.cpp", "reorder.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         # packed-fp32 VALU forms are switched off for device code on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # MFMA accumulators stay in ordinary VGPRs: with the AGPR form the register allocator
         # copies the accumulators of the unrolled fragment ring back and forth on every round
         "-mllvm", "-amdgpu-mfma-vgpr-form=1",
         "-Wall", "-Wextra", "-Wno-unused-command-line-argument"]


def sources() -> list[str]:
    return [os.path.join(CSRC, s) for s in SOURCES]


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp")]
    deps.append(os.path.join(HERE, "..", "include", "rsh_spmm.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True) -> str:
    if force or needs_build():
        cmd = [HIPCC, *FLAGS, "-o", LIB, *sources(), "-lpthread"]
        subprocess.check_call(cmd)
    return LIB
