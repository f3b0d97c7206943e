"""Builds libtc.so (HIP kernels + host runtime) for gfx950 with hipcc, in-tree."""

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtc.so")
SOURCES = ["tc_planner.cpp", "tc_runtime.cpp", "tc_dispatch.cpp", "tc_io.cpp", "tc_movers.cpp", "tc_kernels.hip"]


def build(verbose: bool = True) -> str:
    """Compile every source for gfx950 and link libtc.so next to this file."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc, "-x", "hip", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-command-line-argument",
               "-I", os.path.join(ROOT, "include"), "-I", CSRC,
               "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        objs.append(obj)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", "-o", LIB] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    build_c_example(verbose)
    return LIB


def build_c_example(verbose: bool = True) -> str:
    """The plain-C99 users of the ABI under tests/c (run by the GPU tests): built with gcc
    against include/tc.h and the HIP runtime API, libtc.so found at run time next to them."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    out = ""
    for name in ("tc_opt_example", "tc_example"):
        src = os.path.join(ROOT, "tests", "c", name + ".c")
        out = os.path.join(ROOT, "tests", "c", name + ".bin")
        cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror", "-D__HIP_PLATFORM_AMD__",
               "-I", os.path.join(ROOT, "include"), "-I", os.path.join(rocm, "include"), src, "-o", out,
               "-L", HERE, "-l:libtc.so", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
               "-Wl,-rpath,$ORIGIN/../../paper_2511_14124_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
    return out


if __name__ == "__main__":
    build()
    sys.exit(0)
