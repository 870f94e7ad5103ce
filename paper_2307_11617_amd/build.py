"""Builds librfast.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "librfast.so")
SOURCES = ["rfast_api.cpp", "rfast_resolve.hip", "rfast_round.hip", "rfast_block.hip", "rfast_wave.hip", "rfast_grad.hip", "rfast_softmax.hip",
           "rfast_diag.hip", "rfast_schedule.hip"]
# no floating-point contraction: the two kernels that implement the separable round must round alike
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-shared", "-std=c++17", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False) -> str:
    cmd = ["hipcc", *FLAGS, "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"), "-o", LIB]
    cmd += [os.path.join(PKG, "csrc", s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout + res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building librfast.so")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
