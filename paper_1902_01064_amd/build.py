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


def build_asan_driver():
    """tests/_bin/gpu_asan_driver: the C ABI's host code (hop_api.cpp, hop_sim.cpp) under AddressSanitizer and
    UBSan, linked with the product's kernel object; tests/test_gpu_asan_driver.py runs it on a GPU.  Host code
    only is instrumented; call after build_library()."""
    import shutil
    gxx = shutil.which("g++")
    if gxx is None:
        print("build_asan_driver: no g++, skipped", flush=True)
        return None
    out_dir = os.path.join(ROOT, "tests", "_bin")
    os.makedirs(out_dir, exist_ok=True)
    exe = os.path.join(out_dir, "gpu_asan_driver")
    _run([gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
          "-ffp-contract=off", "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include", "-I", os.path.join(ROOT, "include"),
          "-I", CSRC, os.path.join(ROOT, "tests", "gpu_driver.cpp"), os.path.join(CSRC, "hop_api.cpp"),
          os.path.join(CSRC, "hop_sim.cpp"), os.path.join(OBJ, "hop_kernels.hip.o"),
          "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-o", exe])
    return exe


if __name__ == "__main__":
    build_library()
    build_asan_driver()
    sys.exit(0)
