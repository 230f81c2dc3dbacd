"""Compiles the HIP sources of this package for gfx950 into in-tree shared libraries.

Two libraries come out of the same sources: the product build (bf16 activations, MFMA kernels)
and the fp32 debug build (float activations, plain kernels) used to separate kernel-logic errors
from bf16 rounding.
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
SOURCES = ["instance.hip", "zigzag.hip", "plan.hip", "k_small.hip", "k_gemm.hip", "k_attn.hip"]
LIB = os.path.join(PKG, "libblitzlayer.so")
LIB_FP32 = os.path.join(PKG, "libblitzlayer_fp32dbg.so")

COMMON = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-result",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


def _compile(out: str, extra) -> None:
    cmd = [_hipcc()] + COMMON + list(extra) + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the packed-fp32 device feature and says so; everything else is shown
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        sys.stderr.write(err + "\n")
        raise RuntimeError("hipcc failed for " + out)
    if err.strip():
        sys.stderr.write(err + "\n")


def build_all(debug_too: bool = True) -> None:
    _compile(LIB, [])
    if debug_too:
        _compile(LIB_FP32, ["-DBZ_FP32_DEBUG"])


if __name__ == "__main__":
    build_all()
    print("built", LIB, "and", LIB_FP32)
