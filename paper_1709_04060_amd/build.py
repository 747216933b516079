"""Builds libbsgemm.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libbsgemm.so")

SOURCES = ["bs_pack.hip", "bs_gemm.hip", "bs_gemm_w1.hip", "bs_gemm_w2.hip", "bs_gemm_w3.hip", "bs_gemm_w4.hip", "bs_gemv.hip", "bs_gemv_w1.hip", "bs_gemv_w2.hip", "bs_gemv_w3.hip", "bs_gemv_w4.hip", "bs_planes_mfma.hip",
           "bs_threshold.hip", "bs_im2col.hip", "bs_pool.hip", "bs_dense.hip", "bs_probe.hip", "bs_streamline.cpp", "bs_misc.cpp"]

# -packed-fp32-ops is switched off on purpose: this code has no float math, and the
# packed FP32 forms are not to be generated on this target.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + INCLUDE, "-I" + CSRC,
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def _compile(src: str, extra: list[str]) -> str:
    obj = os.path.join(OBJDIR, os.path.splitext(src)[0] + ".o")
    lang = ["-x", "hip"] if src.endswith(".cpp") else []
    cmd = [_hipcc()] + HIPCC_FLAGS + extra + lang + ["-c", os.path.join(CSRC, src), "-o", obj]
    subprocess.check_call(cmd)
    return obj


def build(verbose: bool = False, extra_flags: list[str] | None = None, jobs: int = 8) -> str:
    """Compile every source and link libbsgemm.so.  Always recompiles."""
    os.makedirs(OBJDIR, exist_ok=True)
    extra = list(extra_flags or [])
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra), SOURCES))
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
