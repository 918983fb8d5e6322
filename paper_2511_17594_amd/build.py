"""Builds libautosage.so (gfx950) in-tree from csrc/ with hipcc.

hipcc cross-compiles for gfx950 without a GPU.  The library is placed next to this
file so that it travels with the source tree; nothing is installed anywhere else.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libautosage.so")

SOURCES = [
    "api.cpp", "selector.cpp", "plan.hip", "softmax.hip",
    "spmm.hip", "spmm_f32.hip", "spmm_bf16.hip", "spmm_f16.hip",
    "sddmm.hip", "sddmm_f32.hip", "sddmm_bf16.hip", "sddmm_f16.hip",
    "attention.hip", "attention_f32.hip", "attention_bf16.hip", "attention_f16.hip", "transpose.hip", "stream_probe.hip",
    "static_scratch.hip",
]

# -packed-fp32-ops is switched off on purpose: packed fp32 instructions are not to be generated.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *HIPCC_FLAGS, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, res.stderr[-4000:]))
    return obj


def build_library(jobs: int = 8, verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n%s" % res.stderr[-4000:])
    if verbose:
        print("built", LIB, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    build_library(verbose=True)
