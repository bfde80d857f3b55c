"""Builds libelixir_chunk.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_PKG, "csrc")
LIB = os.path.join(_PKG, "libelixir_chunk.so")
SOURCES = ["ctx.cpp", "layout.cpp", "offload.cpp", "pack.hip", "reduce.hip", "norm.hip", "adam.hip"]
HOST_SOURCES = ["host_adam.cpp", "benefit.cpp", "rcache_sim.cpp", "arena.cpp"]   # plain C++ (x86 intrinsics, threads): compiled by g++, linked into the same library

# -ffp-contract=off: fused multiply-adds appear only where the source asks for them, so the
#   separately rounded multiply/add of the gradient reduction stay separate.
# -packed-fp32-ops off: keeps the compiler from forming packed fp32 instructions.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-mllvm", "-amdgpu-kernarg-preload-count=16",
               "-Wall", "-Wno-unused-command-line-argument"]


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + f".tmp{os.getpid()}"
    objs = []
    for src in HOST_SOURCES:
        obj = os.path.join(CSRC, src + f".{os.getpid()}.o")
        cmd = ["g++", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fno-fast-math", "-pthread", "-Wall", "-c",
               os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        objs.append(obj)
    try:
        cmd = [hipcc, *HIPCC_FLAGS, "-x", "hip", *[os.path.join(CSRC, s) for s in SOURCES], "-x", "none", *objs, "-pthread", "-o", tmp]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
    finally:
        for o in objs:
            if os.path.exists(o):
                os.remove(o)
    os.replace(tmp, LIB)
    return LIB


def build_synth(verbose: bool = False) -> str:
    """The device-side twin of the seeded input generator (harness code, separate library)."""
    root = os.path.dirname(_PKG)
    src = os.path.join(root, "synth", "gen.hip")
    out = os.path.join(root, "synth", "libsynth_gen.so")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = out + f".tmp{os.getpid()}"
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument", src, "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, out)
    return out


def ensure_built(verbose: bool = False) -> None:
    """Builds what is missing and nothing else: callers that only want to run (tests, the smoke check, the
    benchmark) load the libraries that are there and compile only when there are none."""
    if not os.path.exists(LIB):
        build_library(verbose)
    if not os.path.exists(os.path.join(os.path.dirname(_PKG), "synth", "libsynth_gen.so")):
        build_synth(verbose)


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_synth(verbose=True))
