"""Builds libsprinter.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libsprinter.so")
SOURCES = ["kernels.hip", "mega.hip", "abi.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         # packed-fp32 VALU forms are kept off on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def build_library(verbose: bool = True) -> str:
    cmd = ["hipcc", *FLAGS, "-x", "hip", *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                    if "packed-fp32-ops' is not a recognized feature" not in l)
    if out.strip() and verbose:
        print(out, flush=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return LIB


if __name__ == "__main__":
    build_library()
    print("built", LIB)
    sys.exit(0)
