"""Builds libganq.so (the C-ABI library with the gfx950 kernels) in-tree with hipcc.

    python -m paper_2501_12956_amd.build

Each .hip source is compiled to an object file in ``_build/`` and the objects
are linked into ``paper_2501_12956_amd/libganq.so``.  hipcc cross-compiles for
gfx950 without a GPU present.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
BUILD = os.path.join(ROOT, "_build")
LIB = os.path.join(PKG, "libganq.so")

SOURCES = ["ganq_api.hip", "gemm_f32.hip", "hessian.hip", "cholesky.hip", "init_codebooks.hip",
           "update_s.hip", "update_t.hip", "loss.hip", "outlier_split.hip", "gemm_split.hip",
           "lut_gemv.hip", "peaks.hip"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed fp32 VALU forms are kept off for every kernel in this library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src):
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, res.stdout, res.stderr))
    return obj


def build(verbose=True, jobs=8):
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(_compile, SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (res.stdout, res.stderr))
    if verbose:
        print("built", LIB)
    return LIB


def build_sanitized(outdir, jobs=8):
    """A copy of the library whose HOST code carries AddressSanitizer and UndefinedBehaviorSanitizer
    instrumentation (device code is compiled as usual but at -O1: it is never run), for checking the
    argument validation of the C ABI on a machine without a GPU.  Returns the path of the library."""
    os.makedirs(outdir, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    flags = [f if f != "-O3" else "-O1" for f in FLAGS] + san

    def one(src):
        obj = os.path.join(outdir, os.path.splitext(src)[0] + ".o")
        res = subprocess.run([_hipcc(), *flags, "-c", os.path.join(CSRC, src), "-o", obj],
                             capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, res.stdout, res.stderr))
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(one, SOURCES))
    lib = os.path.join(outdir, "libganq_san.so")
    res = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address",
                          "-fsanitize=undefined", "-Wno-option-ignored", "-o", lib, *objs],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (res.stdout, res.stderr))
    return lib


if __name__ == "__main__":
    build()
    sys.exit(0)
