"""Builds libiflow.so (the C-ABI library of include/iflow.h) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libiflow.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -ffp-contract=off: the quantizer's arithmetic must not be fused (fused multiply-adds are written out
#   explicitly where they are wanted).
# -packed-fp32-ops off: the compiler is kept from forming packed fp32 instructions.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]
# The first kernel arguments arrive in scalar registers at wavefront start instead of through a scalar load
# (the GEMV kernel puts what it needs to form its first addresses there); worth 1-2 % on the 8 MiB matrices.
FLAGS += ["-mllvm", "-amdgpu-kernarg-preload-count=16"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_lib(verbose: bool = False) -> str:
    """Compile every HIP source into paper_2401_08294_amd/libiflow.so (always recompiles)."""
    cmd = [HIPCC] + FLAGS + sources() + ["-o", LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
