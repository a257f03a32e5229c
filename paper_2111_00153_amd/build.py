"""Builds librmsmp.so (hipcc, gfx950 only) next to this file."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "librmsmp.so")
SOURCES = ["csrc/pack_host.cpp", "csrc/kernels.hip", "csrc/fakequant.hip", "csrc/api.hip"]
HEADERS = ["csrc/rmsmp_internal.h", "../include/rmsmp.h"]


def hipcc_command():
    return (["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
             # packed-FP32 VALU forms are kept off (per-lane fp32 epilogue must be bit-reproducible)
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-ffp-contract=off", "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc")]
            + [os.path.join(HERE, s) for s in SOURCES] + ["-o", LIB])


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(HERE, f)) > t for f in SOURCES + HEADERS)


def build_library(force=True):
    """Compile the library.  force=False only compiles when the .so is missing."""
    if force or not os.path.exists(LIB):
        subprocess.check_call(hipcc_command(), cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build_library())
