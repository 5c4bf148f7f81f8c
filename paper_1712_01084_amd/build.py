"""Builds the C-ABI library (libpivotfc.so) in-tree with hipcc for gfx950.

Run as ``python -m paper_1712_01084_amd.build``.  hipcc cross-compiles, so no
GPU is needed to build.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libpivotfc.so")

SOURCES = ["pivot_gemv_f32.hip", "pivot_gemv_f16.hip", "pivot_mfma_f16.hip", "pivot_mfma_lds_f16.hip", "pivot_mfma_xrow_f16.hip", "pivot_colmajor.hip", "pivot_misc.hip", "pivot_lstm_persist.hip", "pivot_mlp_persist.hip", "pivot_launch.hip", "pivot_static.hip",
           "pivot_plan.cpp", "pivot_search.cpp", "pivot_api.cpp"]

COMMON = ["-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
          "-Wall", "-Wno-unused-function"]
# packed fp32 instructions are kept off for every device compile
# the leading kernel arguments are preloaded into SGPRs (up to 14 dwords on gfx950)
# the device code of every object is stored compressed (the library is 3 MB instead of 14; the runtime unpacks
# a code object when the library is loaded)
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-mllvm", "-amdgpu-kernarg-preload-count=16", "--offload-compress"]


def _hipcc():
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


def _compile(src, objdir=None, device_flags=None):
    objdir = objdir or OBJDIR
    obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc()] + COMMON + (DEVICE if device_flags is None else device_flags) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("compile failed: %s\n%s" % (" ".join(cmd), out))
    return obj, out


def build(verbose=False, out=None, objdir=None, device_flags=None, only=None):
    """Compiles every source and links the shared library.  ``out``, ``objdir``
    and ``device_flags`` let an experiment build a variant beside the product;
    with ``only`` (a list of sources) just those are compiled with the variant's
    flags and every other object is taken from the product build."""
    objdir = objdir or OBJDIR
    os.makedirs(objdir, exist_ok=True)

    def one(src):
        if only is not None and src not in only:
            obj = os.path.join(OBJDIR, os.path.splitext(src)[0] + ".o")
            if not os.path.exists(obj):
                raise RuntimeError("%s missing: build the product first" % obj)
            return obj, ""
        return _compile(src, objdir, device_flags)

    with ThreadPoolExecutor(max_workers=8) as ex:
        results = list(ex.map(one, SOURCES))
    if verbose:
        for _, log in results:
            if log.strip():
                print(log)
    objs = [o for o, _ in results]
    out = out or LIB
    cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", out] + objs + ["-Wl,-rpath,/opt/rocm/lib"]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed: %s\n%s" % (" ".join(cmd), r.stdout))
    return out


if __name__ == "__main__":
    print(build(verbose=True))
