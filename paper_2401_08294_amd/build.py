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
# Measurement builds: extra -D options from the environment (e.g. IFLOW_HIPCC_DEFINES="-DIFLOW_CHAIN_ABL=1"); the library's
# own build passes none.
FLAGS += os.environ.get("IFLOW_HIPCC_DEFINES", "").split()


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _run(cmd):
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + err)
    return err


def build_lib(verbose: bool = False) -> str:
    """Compile every HIP source into paper_2401_08294_amd/libiflow.so (always recompiles): one object per source, the
    sources side by side on up to eight host threads, then one link."""
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in FLAGS if f != "-shared"]
    srcs = sources()
    objs = [os.path.join(objdir, os.path.basename(s)[:-4] + ".o") for s in srcs]
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as pool:
        errs = list(pool.map(lambda so: _run([HIPCC] + compile_flags + ["-c", so[0], "-o", so[1]]), zip(srcs, objs)))
    errs.append(_run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB]))
    if verbose:
        for e in errs:
            if e.strip():
                print(e)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
