"""Builds librfast.so (hand-written HIP for gfx950) in-tree with hipcc.

Every source is compiled to an object of its own (in parallel) and the objects are linked;
`build()` recompiles everything, `build(incremental=True)` only what changed."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "librfast.so")
OBJ = os.path.join(PKG, "_build")
SOURCES = ["rfast_api.cpp", "rfast_resolve.hip", "rfast_round.hip", "rfast_block.hip", "rfast_wave.hip", "rfast_grad.hip", "rfast_softmax.hip",
           "rfast_diag.hip", "rfast_schedule.hip", "rfast_tiny.hip"]
# no floating-point contraction: the kernels that implement the separable round must round alike
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _newest_header() -> float:
    t = 0.0
    for d in (os.path.join(PKG, "csrc"), os.path.join(ROOT, "include")):
        for f in os.listdir(d):
            if f.endswith(".h"):
                t = max(t, os.path.getmtime(os.path.join(d, f)))
    return t


def _compile(src: str, incremental: bool, header_time: float):
    path = os.path.join(PKG, "csrc", src)
    obj = os.path.join(OBJ, src + ".o")
    if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(path), header_time):
        return obj, 0, ""
    cmd = ["hipcc", *FLAGS, "-x", "hip", "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"), "-c", path, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    return obj, res.returncode, res.stdout + res.stderr


def build(verbose: bool = False, incremental: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    header_time = _newest_header()
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        done = list(pool.map(lambda s: _compile(s, incremental, header_time), SOURCES))
    for obj, rc, text in done:
        if verbose or rc != 0:
            print(text)
        if rc != 0:
            raise RuntimeError(f"hipcc failed compiling {obj}")
    res = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *[o for o, _, _ in done]],
                         capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout + res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed linking librfast.so")
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose="-v" in sys.argv, incremental="--all" not in sys.argv))
