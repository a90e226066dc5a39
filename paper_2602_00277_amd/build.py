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

SOURCES = ["ftar_reduce.hip", "ftar_ring.hip", "ftar_persistent.hip", "ftar_probe.hip", "ftar_api.cpp"]
HEADERS = ["ftar_internal.h", "ftar_device.h"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
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
    deps = sources() + [os.path.join(CSRC, h) for h in HEADERS] + [os.path.join(ROOT, "include", "ftar.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose=True):
    """Compiles every source to an object file (all at once: the files are independent) and links."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)
    jobs = []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        cmd = [hipcc] + FLAGS + ["-x", "hip", "-c", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", obj, src]
        if verbose:
            print(" ".join(cmd), flush=True)
        jobs.append((cmd, obj, subprocess.Popen(cmd)))
    failed = [cmd for cmd, _, p in jobs if p.wait() != 0]
    if failed:
        raise subprocess.CalledProcessError(1, failed[0])
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + [obj for _, obj, _ in jobs]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
