"""Builds libmoska.so (HIP, gfx950) in-tree with hipcc.  Run: python -m paper_2511_06010_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libmoska.so")
SOURCES = ["attn_mfma_shared_bf16.hip", "attn_mfma_shared_fp8.hip", "attn_mfma.hip", "api.hip", "route.hip",
           "bucket.hip", "attn_generic.hip", "merge.hip", "cache_build.hip"]
# packed-fp32 VALU forms are disabled on purpose (they have produced wrong results on the test machines)
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-parameter",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


# The MFMA attention kernels never produce or consume a NaN (empty key sets are handled by explicit
# -inf tests, infinities stay honoured), and saying so lets the softmax take its row maxima with
# v_max3_f32 instead of first quieting every MFMA result (14 instead of 34 instructions per tile).
PER_SOURCE = {s: ["-fno-honor-nans"] for s in ("attn_mfma_shared_bf16.hip", "attn_mfma_shared_fp8.hip", "attn_mfma.hip")}


def _compile(src: str, extra) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    subprocess.check_call(["hipcc", *FLAGS, *PER_SOURCE.get(src, []), *extra, "-c", os.path.join(CSRC, src), "-o", obj])
    return obj


def build_library(extra_flags=(), verbose: bool = True) -> str:
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build_library(sys.argv[1:])
