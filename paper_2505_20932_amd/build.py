"""Builds libcwac_hip.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
BUILD = os.path.join(ROOT, "_build")
LIB = os.path.join(PKG, "libcwac_hip.so")

SOURCES = ["status.hip", "quantize.hip", "calib_stats.hip", "fold_epilogue.hip", "qlinear_forward.hip", "qlinear_fast.hip",
           "probe.hip", "w4a16.hip", "block_glue.hip"]

# -ffp-contract=off: the epilogue and the fold are defined as sequences of single
# roundings; packed fp32 instructions are disabled for the device pass.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _hipcc() -> str:
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _compile(src: str, extra=(), suffix: str = "") -> str:
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + suffix + ".o")
    cmd = [_hipcc(), *HIPCC_FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    subprocess.run(cmd, check=True, stderr=subprocess.PIPE, text=True)
    return obj


def build_library(verbose: bool = True) -> str:
    os.makedirs(BUILD, exist_ok=True)
    try:
        with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
            objs = list(ex.map(_compile, SOURCES))
        subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB],
                       check=True, stderr=subprocess.PIPE, text=True)
    except subprocess.CalledProcessError as e:
        sys.stderr.write(e.stderr or "")
        raise
    if verbose:
        print(f"built {LIB}")
    return LIB


STAMP_LIB = os.path.join(PKG, "libcwac_hip_timeline.so")


def build_timeline_library(verbose: bool = True) -> str:
    """Development build for `bench.py --tile-timeline`: the same library with the forward kernels
    compiled with -DCWAC_V_STAMP, which makes every wavefront of the direct-to-LDS kernels record
    100 MHz time stamps at five points of each tile and exports cwac_debug_stamps to read them.
    Never loaded by the product path (binding.lib() loads libcwac_hip.so)."""
    build_library(verbose=False)
    try:
        obj = _compile("qlinear_fast.hip", extra=("-DCWAC_V_STAMP",), suffix="_timeline")
        others = [os.path.join(BUILD, os.path.splitext(f)[0] + ".o") for f in SOURCES if f != "qlinear_fast.hip"]
        subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *others, obj, "-o", STAMP_LIB],
                       check=True, stderr=subprocess.PIPE, text=True)
    except subprocess.CalledProcessError as e:
        sys.stderr.write(e.stderr or "")
        raise
    if verbose:
        print(f"built {STAMP_LIB}")
    return STAMP_LIB


if __name__ == "__main__":
    if "--timeline" in sys.argv[1:]:
        build_timeline_library()
    else:
        build_library()
