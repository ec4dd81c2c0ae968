"""Builds libsquat.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2503_24358_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(ROOT, "_build")
LIB = os.path.join(PKG, "libsquat.so")

SOURCES = ["squat_api.cpp", "squat_quantize.hip", "squat_quantize_pc.hip", "squat_dequantize.hip",
           "squat_subspace.hip", "squat_prepare.hip", "squat_scores.hip", "squat_scores_pc.hip", "squat_scores_rope.hip",
           "squat_cache.hip"]

# Packed-fp32 VALU ops are switched off on purpose: some of their forms have given wrong results on this
# hardware now and then, silently; the kernels' vector budget is therefore 64 lanes per CU and clock.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


# Per-file extras.  The scores kernels read every matrix-product result right away with ordinary vector
# instructions: keep those results in the ordinary register file instead of the accumulation registers
# (saves one copy per result register).  The update-matrix kernel for up to 64 subspace directions keeps 64
# unknowns per lane in registers through two triangular substitutions written as fully unrolled loops: past the
# compiler's default size limit for such loops it leaves them rolled and the unknowns in scratch memory.
EXTRA = {"squat_scores.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
         "squat_scores_pc.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
         "squat_scores_rope.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
         "squat_prepare.hip": ["-mllvm", "-pragma-unroll-threshold=200000"]}


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *FLAGS, *EXTRA.get(src, []), "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, res.stderr[-4000:]))
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr[-4000:])
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
