"""Build libtperm.so (host planner + HIP kernels for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtperm.so")
PROBE = os.path.join(HERE, "pattern_probe")
LATENCY_PROBE = os.path.join(HERE, "latency_probe")
SOURCES = ["plan.cpp", "model.cpp", "api.cpp", "cache.cpp", "kernels.hip", "verify.hip", "tile_inst_u64_256.hip", "tile_inst_u32_256.hip",
           "tile_inst_u64_64.hip", "tile_inst_u32_64.hip", "tile_inst_big_u64.hip", "tile_inst_big_u32.hip"]
HEADERS = ["pattern_probe.hip", "latency_probe.hip", "plan.hpp", "kernels.hpp", "verify.hpp", "tperm_desc.h", "tile_kernel.hpp", os.path.join("..", "..", "include", "tperm.h"),
           os.path.join("..", "..", "include", "tperm_tuning.h")]

# -packed-fp32-ops is switched off for all device code built here (no packed FP32
# instructions are wanted from the compiler; the kernels only move bits anyway).
COMMON_FLAGS = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra", "-Wno-unused-parameter"]
HOST_FLAGS = ["-x", "c++", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include"]   # planner, C ABI
DEVICE_FLAGS = ["-x", "hip", "--offload-arch=gfx950",
                "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every source for gfx950 and link the shared library."""
    if not force and not needs_build():
        return LIB
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        lang = DEVICE_FLAGS if src.endswith(".hip") else HOST_FLAGS
        cmd = [hipcc(), *COMMON_FLAGS, *lang, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd)))
        objs.append(obj)
    for cmd, p in procs:
        if p.wait() != 0:
            raise RuntimeError("compile failed: " + " ".join(cmd))
    cmd = [hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    # the pattern probe: a stand-alone measurement tool (what a transpose tile's access pattern
    # can reach on this memory system, whatever kernel issues it)
    cmd = [hipcc(), *COMMON_FLAGS, *DEVICE_FLAGS, os.path.join(CSRC, "pattern_probe.hip"), "-o", PROBE]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    # the latency probe: pointer-chasing measurement of the machine constants the analytical
    # model takes (memory and LDS latency, departure delay)
    cmd = [hipcc(), *COMMON_FLAGS, *DEVICE_FLAGS, os.path.join(CSRC, "latency_probe.hip"), "-o", LATENCY_PROBE]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--if-needed" not in sys.argv, verbose=True))
