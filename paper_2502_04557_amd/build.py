"""Builds libsprinter.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libsprinter.so")
NATIVE_BENCH = os.path.join(PKG, "native_bench")
SOURCES = ["k_norm.hip", "k_gemm.hip", "k_attn.hip", "k_lmhead.hip", "k_control.hip", "k_sd.hip", "abi.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed-fp32 VALU forms are kept off on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                    if "packed-fp32-ops' is not a recognized feature" not in l)
    if out.strip() and verbose:
        print(out, flush=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)


def build_library(verbose: bool = True) -> str:
    """Every source is compiled (in parallel) on each call, then linked into the shared library."""
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = [os.path.join(objdir, s + ".o") for s in SOURCES]
    cmds = [["hipcc", *FLAGS, "-x", "hip", "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=len(cmds)) as ex:
        list(ex.map(lambda c: _run(c, verbose), cmds))
    _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], verbose)
    # the Python-free runner of dumped workloads (hardware-counter runs); it only uses the public C ABI
    _run(["hipcc", *FLAGS, "-x", "hip", os.path.join(CSRC, "native_bench.cpp"), "-L" + PKG, "-lsprinter",
          "-Wl,-rpath,$ORIGIN", "-o", NATIVE_BENCH], verbose)
    return LIB


if __name__ == "__main__":
    build_library()
    print("built", LIB)
    sys.exit(0)
