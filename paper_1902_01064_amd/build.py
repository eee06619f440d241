"""Builds csrc/ into libhop.so next to this file with hipcc for gfx950.

`python -m paper_1902_01064_amd.build` compiles every time it is called; the
binding only loads what is already built.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhop.so")
OBJ = os.path.join(HERE, "_build")

COMMON = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC]
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-munsafe-fp-atomics"]


def _run(cmd):
    print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)


def build_library():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    objs = []
    for src, extra in (("hop_kernels.hip", DEVICE),
                       ("hop_api.cpp", []),
                       ("hop_sim.cpp", ["-ffp-contract=off"])):
        o = os.path.join(OBJ, src + ".o")
        _run([hipcc] + COMMON + extra + ["-c", os.path.join(CSRC, src), "-o", o])
        objs.append(o)
    _run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950"] + objs + ["-o", LIB])
    return LIB


if __name__ == "__main__":
    build_library()
    sys.exit(0)
