"""Build the HIP library in-tree (``librsh.so`` next to this file) for gfx950."""
from __future__ import annotations

import hashlib
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


STAMP = LIB + ".sources"   # digest of the sources and flags the library was built from


def source_digest() -> str:
    deps = sources() + sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp"))
    deps.append(os.path.join(HERE, "..", "include", "rsh_spmm.h"))
    h = hashlib.sha256(" ".join(FLAGS).encode())
    for d in deps:
        with open(d, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def needs_build() -> bool:
    """True when there is no library or it was built from other sources (compared by content, so
    that a copy of the tree with new file times is not taken for an edit)."""
    if not os.path.exists(LIB) or not os.path.exists(STAMP):
        return True
    with open(STAMP) as f:
        return f.read().strip() != source_digest()


def build(force: bool = True) -> str:
    if force or needs_build():
        cmd = [HIPCC, *FLAGS, "-o", LIB, *sources(), "-lpthread"]
        subprocess.check_call(cmd)
        with open(STAMP, "w") as f:
            f.write(source_digest() + "\n")
    return LIB
