"""Builds libfusco.so (HIP kernels + C boundary) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "fusco.hip")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(HERE, "libfusco.so")


def hipcc_path() -> str:
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def build_library(verbose: bool = False) -> str:
    """Compile the library; always recompiles.  Returns the path of the shared object."""
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           # packed fp32 instructions are kept out of the generated code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument",
           "-I", INCLUDE, "-o", tmp, SRC, "-Wl,-rpath,/opt/rocm/lib"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out, flush=True)
    os.replace(tmp, LIB)
    return LIB


EXAMPLE_SRC = os.path.join(ROOT, "examples", "c_abi_usage.c")
EXAMPLE_BIN = os.path.join(ROOT, "examples", "c_abi_usage")


def build_c_example(verbose: bool = False) -> str:
    """Compile the plain-C user of the boundary (host compiler only) against the built library."""
    rocm = os.path.dirname(os.path.dirname(os.path.realpath(hipcc_path())))
    if not os.path.isdir(os.path.join(rocm, "include", "hip")):
        rocm = "/opt/rocm"
    cmd = ["gcc", "-std=c99", "-Wall", "-O1", EXAMPLE_SRC, "-I", INCLUDE, "-I", os.path.join(rocm, "include"),
           "-D__HIP_PLATFORM_AMD__", "-L", HERE, "-lfusco", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../paper_2512_22036_amd", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", EXAMPLE_BIN]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return EXAMPLE_BIN


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_c_example(verbose=True))
