"""Builds libftar.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc.

Run `python -m paper_2602_00277_amd.build` after changing anything under csrc/
or include/.  hipcc cross-compiles, so no GPU is needed to build.
"""
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libftar.so")

SOURCES = ["ftar_kernels.hip", "ftar_api.cpp"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                      # no fused multiply-add: additions and the scale stay separate roundings
    "-fno-gpu-flush-denormals-to-zero",            # fp32 denormals are kept, as on the host
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + [os.path.join(CSRC, "ftar_internal.h"), os.path.join(ROOT, "include", "ftar.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose=True):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", LIB] + sources()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
