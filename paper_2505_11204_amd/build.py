"""Build ``librandes.so`` (gfx950) in-tree with hipcc.

``python -m paper_2505_11204_amd.build`` compiles the sources under
``csrc/`` into ``paper_2505_11204_amd/librandes.so``.  hipcc cross-compiles, so
no GPU is needed to build.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librandes.so")
SOURCES = ["kernels.hip", "lora.hip", "noalloc.hip", "plan.cpp", "api.cpp", "place.cpp"]
HEADERS = ["launch.hpp", "plan.hpp", "philox.hpp", "device_util.hpp", "api_internal.hpp",
           os.path.join("..", "..", "include", "randes.h"), os.path.join("..", "..", "include", "randes_bench.h"),
           os.path.join("..", "..", "include", "randes_place.h")]

# -ffp-contract=off: the merge is adds only and the retrieve asks for its one fused
# multiply-add explicitly, so nothing may be contracted behind the source's back.
# packed-fp32 instructions are disabled for the device code.
COMMON = ["-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-Wall", "-Wextra", "-Wno-unused-parameter"]
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    files = [os.path.join(CSRC, s) for s in SOURCES + HEADERS] + [os.path.abspath(__file__)]
    return any(os.path.getmtime(f) > t for f in files)


def build(force=True, verbose=False, extra=()):
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for s in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(s)[0] + ".o")
        if s.endswith(".hip"):
            cmd = [hipcc, "-c", os.path.join(CSRC, s), "-o", obj] + COMMON + DEVICE + list(extra)
        else:  # host-only translation units: plain g++ against the HIP runtime API header
            cmd = ["g++", "-c", os.path.join(CSRC, s), "-o", obj, "-I/opt/rocm/include",
                   "-D__HIP_PLATFORM_AMD__"] + COMMON
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd)))
        objs.append(obj)
    for cmd, p in procs:
        if p.wait() != 0:
            raise RuntimeError("compile failed: " + " ".join(cmd))
    link = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return LIB


if __name__ == "__main__":
    build(force=True, verbose=True, extra=sys.argv[1:])
    print("built", LIB)
