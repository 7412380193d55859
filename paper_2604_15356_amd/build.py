"""Builds libplc.so (gfx950) in-tree.

Every HIP source is compiled in two passes, device then host, so that the flag that keeps the
compiler from forming packed fp32 instructions reaches the device pass alone (the host target does not
know the feature).  The device pass leaves a bundled code object that the host pass embeds; sources are
compiled side by side and linked at the end.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libplc.so")
HIP_SOURCES = ["plc_api.hip", "plc_predict.hip", "plc_hist_freq.hip", "plc_rans.hip", "plc_index.hip",
               "plc_linear.hip"]
CXX_SOURCES = ["plc_trie.cpp"]
COMMON = ["-O3", "-std=c++17", "-Wall", "-I", os.path.join(ROOT, "include"), "-I", CSRC]
# The coders read and write their LDS stages and packed rows through pointers of several types; the order of
# those accesses must not depend on what the compiler concludes from the types.  (Not for the contraction: its
# LDS is filled by the memory system and read as one type, and the flag costs its loop a quarter of its rate.)
NO_STRICT_ALIASING = {"plc_predict.hip", "plc_hist_freq.hip", "plc_rans.hip", "plc_index.hip"}
ARCH = "--offload-arch=gfx950"
DEVICE_ONLY = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)


def _compile_hip(clang, src, out_dir, verbose):
    base = os.path.join(out_dir, os.path.splitext(os.path.basename(src))[0])
    fatbin, obj = base + ".hipfb", base + ".o"
    extra = ["-fno-strict-aliasing"] if os.path.basename(src) in NO_STRICT_ALIASING else []
    _run([clang, "-x", "hip", ARCH, "--offload-device-only", "--gpu-bundle-output", *COMMON, *extra, *DEVICE_ONLY,
          "-c", src, "-o", fatbin], verbose)
    _run([clang, "-x", "hip", ARCH, "--offload-host-only", "-fPIC", *COMMON,
          "-Xclang", "-fcuda-include-gpubinary", "-Xclang", fatbin, "-c", src, "-o", obj], verbose)
    return obj


def _compile_cxx(clang, src, out_dir, verbose):
    obj = os.path.join(out_dir, os.path.splitext(os.path.basename(src))[0] + ".o")
    _run([clang, "-fPIC", *COMMON, "-c", src, "-o", obj], verbose)
    return obj


def build(verbose: bool = False) -> str:
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    clang = os.environ.get("HIP_CLANG", os.path.join(rocm, "lib", "llvm", "bin", "clang++"))
    hipcc = os.environ.get("HIPCC", os.path.join(rocm, "bin", "hipcc"))
    out_dir = tempfile.mkdtemp(prefix="plc_build_")
    try:
        jobs = [(_compile_hip, os.path.join(CSRC, s)) for s in HIP_SOURCES]
        jobs += [(_compile_cxx, os.path.join(CSRC, s)) for s in CXX_SOURCES]
        with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
            objs = list(pool.map(lambda j: j[0](clang, j[1], out_dir, verbose), jobs))
        tmp = f"{LIB}.{os.getpid()}.tmp"
        _run([hipcc, ARCH, "-shared", "-fPIC", "-o", tmp, *objs], verbose)
        os.replace(tmp, LIB)
    finally:
        shutil.rmtree(out_dir, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
