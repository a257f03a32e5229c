"""Builds librmsmp.so (hipcc, gfx950 only) next to this file."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "librmsmp.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["csrc/pack_host.cpp", "csrc/gelu_host.cpp", "csrc/kernels.hip", "csrc/patch_wide.hip", "csrc/conv_first.hip", "csrc/fakequant.hip", "csrc/peaks.hip", "csrc/api.hip"]
HEADERS = ["csrc/rmsmp_internal.h", "csrc/device_common.h", "csrc/phase_stamps.h", "csrc/patch_wide.h", "../include/rmsmp.h"]
# (filter taps, channels / 32) families of the wide LDS-resident kernel: csrc/patch_wide_inst.hip is
# compiled once per family so that they build in parallel
WIDE_FAMILIES = [(9, 2), (9, 4), (9, 8), (9, 16), (1, 2), (1, 4), (1, 8), (1, 16), (1, 24)]
# channel counts (in K steps) whose 1x1 family also exists as the variant that stages a deeper layer in parts
WIDE_DEEP_FAMILIES = [16, 24]
WIDE_SOURCE = "csrc/patch_wide_inst.hip"
# channel counts (in K steps) the two-layer launch (a 3x3 and a 1x1 layer on one input) is built for
WIDE_PAIR_FAMILIES = [2, 4, 8]
WIDE_PAIR_SOURCE = "csrc/patch_wide_pair.hip"

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed-FP32 VALU forms are kept off (per-lane fp32 epilogue must be bit-reproducible)
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-ffp-contract=off",
         # leading scalar kernel arguments arrive in registers at wave launch instead of through a
         # first read of the argument block (the wide and the skinny kernels are written for it)
         "-mllvm", "-amdgpu-kernarg-preload-count=14", "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc")]


def _units():
    """(source, extra defines, object path) of every translation unit."""
    units = [(s, [], os.path.join(OBJ_DIR, os.path.splitext(os.path.basename(s))[0] + ".o")) for s in SOURCES]
    for taps, cpt in WIDE_FAMILIES:
        units.append((WIDE_SOURCE, ["-DRMSMP_WIDE_TAPS=%d" % taps, "-DRMSMP_WIDE_CPT=%d" % cpt],
                      os.path.join(OBJ_DIR, "patch_wide_inst_%d_%d.o" % (taps, cpt))))
    for cpt in WIDE_DEEP_FAMILIES:
        units.append((WIDE_SOURCE, ["-DRMSMP_WIDE_TAPS=1", "-DRMSMP_WIDE_CPT=%d" % cpt, "-DRMSMP_WIDE_DEEP=1"],
                      os.path.join(OBJ_DIR, "patch_wide_inst_deep_%d.o" % cpt)))
    for cpt in WIDE_PAIR_FAMILIES:
        units.append((WIDE_PAIR_SOURCE, ["-DRMSMP_WIDE_CPT=%d" % cpt], os.path.join(OBJ_DIR, "patch_wide_pair_%d.o" % cpt)))
    return units


def _compile(unit, extra=()):
    src, defines, obj = unit
    cmd = ["hipcc"] + FLAGS + defines + list(extra) + ["-c", os.path.join(HERE, src), "-o", obj]
    subprocess.check_call(cmd, cwd=HERE)


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(HERE, f)) > t for f in SOURCES + [WIDE_SOURCE, WIDE_PAIR_SOURCE] + HEADERS)


def build_library(force=True, only_changed=False, extra=()):
    """Compile the library: one object per source (in parallel), then one link.

    force=False only compiles when the .so is missing; only_changed=True (a development
    convenience) reuses objects that are newer than their source and every header."""
    if not force and os.path.exists(LIB):
        return LIB
    os.makedirs(OBJ_DIR, exist_ok=True)
    hdr_time = max(os.path.getmtime(os.path.join(HERE, h)) for h in HEADERS)
    todo = []
    for unit in _units():
        src, _, o = unit
        fresh = (only_changed and os.path.exists(o)
                 and os.path.getmtime(o) > max(hdr_time, os.path.getmtime(os.path.join(HERE, src))))
        if not fresh:
            todo.append(unit)
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(todo)))) as ex:
        list(ex.map(lambda u: _compile(u, extra), todo))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC"]
                          + [u[2] for u in _units()] + ["-o", LIB], cwd=HERE)
    return LIB


if __name__ == "__main__":
    import sys
    print(build_library(only_changed="--changed" in sys.argv))
