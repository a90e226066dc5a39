"""Builds libftar.so (HIP kernels + C ABI, include/ftar.h) and the bench-only libftar_measure.so
(bare streaming kernels, include/ftar_measure.h) in-tree for gfx950 with hipcc.

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
MEASURE_LIB = os.path.join(PKG, "libftar_measure.so")

SOURCES = ["ftar_reduce.hip", "ftar_ring.hip", "ftar_persistent.hip", "ftar_api.cpp"]
MEASURE_SOURCES = ["ftar_probe.hip", "ftar_measure.cpp"]      # linked against libftar.so
HEADERS = ["ftar_internal.h", "ftar_device.h"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                      # no fused multiply-add: additions and the scale stay separate roundings
    "-fno-gpu-flush-denormals-to-zero",            # fp32 denormals are kept, as on the host
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES + MEASURE_SOURCES]


def stale():
    if not os.path.exists(LIB) or not os.path.exists(MEASURE_LIB):
        return True
    t = min(os.path.getmtime(LIB), os.path.getmtime(MEASURE_LIB))
    deps = sources() + [os.path.join(CSRC, h) for h in HEADERS] + \
        [os.path.join(ROOT, "include", h) for h in ("ftar.h", "ftar_measure.h")]
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
    measure_objs = {os.path.join(objdir, s + ".o") for s in MEASURE_SOURCES}
    links = [[hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] +
             [obj for _, obj, _ in jobs if obj not in measure_objs],
             [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", MEASURE_LIB] +
             [obj for _, obj, _ in jobs if obj in measure_objs] +
             ["-L", PKG, "-lftar", "-Wl,-rpath,$ORIGIN"]]
    for link in links:
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
