"""Compile the HIP library for gfx950 (in-tree, so the built .so travels with the source tree)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libspd_hip.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build_library(verbose: bool = False, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-o", LIB, os.path.join(CSRC, "spd_api.hip")]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = "is not a recognized feature for this target"   # printed by the host pass for the gfx-only flag
    out = "\n".join(l for l in res.stdout.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{out}")
    if verbose and out.strip():
        print(out)
    return LIB


def build_c_program(verbose: bool = False) -> str:
    """The stand-alone C++ program of tests/host (C ABI + HIP runtime only), linked against the library; a GPU test runs
    it.  Built here so that nothing is compiled on the GPU machine."""
    root = os.path.dirname(PKG)
    src = os.path.join(root, "tests", "host", "abi_gpu_program.cpp")
    exe = os.path.join(root, "tests", "host", "abi_gpu_program")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-I", os.path.join(root, "include"), "-o", exe, src,
           "-L", PKG, "-lspd_hip", "-Wl,-rpath,$ORIGIN/../../paper_2409_19134_amd"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{res.stdout}")
    return exe


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_c_program(verbose=True))
    sys.exit(0)
