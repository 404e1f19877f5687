"""Builds paper_2506_15461_amd/libcheckfree.so (HIP kernels + C ABI) for gfx950.

hipcc cross-compiles without a GPU.  Packed-FP32 instruction selection is
switched off for all device code, and floating-point contraction is off so that
the blend's binary64 operations are rounded one by one.
"""
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libcheckfree.so")
SOURCES = ["cf_kernels.hip", "cf_api.cpp"]


def hipcc_path():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def command(out=LIB, extra=()):
    return [
        hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        "-ffp-contract=off", "-fvisibility=hidden",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wextra", "-Wno-unused-parameter",
        "-I", os.path.join(ROOT, "include"), "-I", CSRC,
        *[os.path.join(CSRC, s) for s in SOURCES],
        *extra,
        "-o", out,
    ]


def build(verbose=True):
    cmd = command()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


C_SMOKE_SRC = os.path.join(ROOT, "tests", "c_abi_smoke.c")
C_SMOKE_BIN = os.path.join(ROOT, "tests", "c_abi_smoke")


def build_c_smoke(verbose=True):
    """The plain-C99 client of the ABI used by the tests (gcc, no HIP compiler)."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-O1", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(ROOT, "include"), "-isystem", os.path.join(rocm, "include"), C_SMOKE_SRC,
           "-o", C_SMOKE_BIN, "-L", PKG, "-lcheckfree", "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../paper_2506_15461_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return C_SMOKE_BIN


if __name__ == "__main__":
    build()
    build_c_smoke()
    sys.exit(0)
