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
HIP_SOURCES = ["cf_kernels.hip", "cf_adam_kernels.hip"]
HOST_SOURCES = ["cf_api.cpp"]


def hipcc_path():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


# hipcc compiles a .hip file once per offload target and once for the host; the host pass does not
# know this device-only feature and says so on stderr (harmless; that exact line is dropped below).
NO_PACKED_FP32 = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
HOST_PASS_NOTE = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"
COMMON = ["-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fvisibility=hidden", "-Wall", "-Wextra",
          "-Wno-unused-parameter", "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def rocm_path():
    return os.environ.get("ROCM_PATH", "/opt/rocm")


def commands(objdir, out=LIB, extra=()):
    """Device code (the .hip files) with packed-FP32 selection off; the host-only C ABI file as plain
    C++ (it has no device code); then the link."""
    hipcc = hipcc_path()
    cmds, objs = [], []
    for src in HIP_SOURCES:
        obj = os.path.join(objdir, src + ".o")
        cmds.append([hipcc, "--offload-arch=gfx950", *COMMON, *NO_PACKED_FP32, *extra, "-c",
                     os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    for src in HOST_SOURCES:
        obj = os.path.join(objdir, src + ".o")
        cmds.append([hipcc, "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-isystem", os.path.join(rocm_path(), "include"),
                     *COMMON, *extra, "-c", os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    cmds.append([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *extra, *objs, "-o", out])
    return cmds


def run(cmd, verbose=True):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    noise = [l for l in r.stderr.splitlines() if l.strip() and l.strip() != HOST_PASS_NOTE]
    if noise:
        print("\n".join(noise), file=sys.stderr, flush=True)
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, cmd)


def build(verbose=True, out=LIB, extra=()):
    import tempfile
    with tempfile.TemporaryDirectory(prefix="cf_build_") as objdir:
        for cmd in commands(objdir, out, extra):
            run(cmd, verbose)
    return out


CEILING_LIB = os.path.join(PKG, "libcf_ceiling.so")


def build_ceiling(verbose=True):
    """The benchmark's two trivial streaming kernels (its independent bandwidth ceilings)."""
    run([hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden",
         "-Wall", "-Wextra", *NO_PACKED_FP32, os.path.join(CSRC, "ceiling_kernels.hip"), "-o", CEILING_LIB], verbose)
    return CEILING_LIB


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
    build_ceiling()
    build_c_smoke()
    sys.exit(0)
