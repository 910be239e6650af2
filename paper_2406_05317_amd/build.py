"""Build step of the HIP library: hipcc for gfx950, in-tree shared object.

    python -m paper_2406_05317_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "liblococo.so")

SOURCES = ["api.cpp", "generic_kernels.hip", "compress_mfma.hip", "attn_mfma.hip", "attn_decode.hip",
           "backward_generic.hip", "tiled_mfma.hip", "peaks.hip"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-fvisibility=hidden", "-Wall", "-Wno-unused-command-line-argument",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


# Per-file extras.  The compression kernel pins its filter slice to the accumulation registers;
# with the VGPR form of the MFMA (accumulators in ordinary registers) nothing is copied between
# the two register halves inside the loop.
EXTRA = {"compress_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form",
                                # the pipeline stages must be unrolled completely (the slices are
                                # selected by compile-time slot numbers); the default size limit of
                                # "#pragma unroll" is too small for the width-21 instantiation
                                "-mllvm", "-pragma-unroll-threshold=200000"],
         # accumulators in ordinary registers: the softmax reads the scores where the MFMA left them
         "attn_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = (["hipcc", "-x", "hip"] + FLAGS + EXTRA.get(src, []) +
           ["-c", os.path.join(CSRC, src), "-o", obj])
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the packed-fp32 feature; that warning is expected
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    """Compile every source and link paper_2406_05317_amd/liblococo.so."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.check_call(cmd)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
