"""TEST INFRASTRUCTURE — ctypes wrapper of the plain-C fp64 oracle
(rfast_oracle_c.c): argument marshalling only.  Used by the tests that
cross-check the two oracles and by the benchmark's cpu_baseline leg."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "rfast_oracle_c.c")
LIB = os.path.join(HERE, "librfast_oracle_c.so")


def build_c_oracle(force: bool = False) -> str:
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        subprocess.run(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", LIB, SRC, "-lm"], check=True)
    return LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        L = C.CDLL(build_c_oracle())
        vp, i32, i64, f64 = C.c_void_p, C.c_int, C.c_int64, C.c_double
        L.rfo_create.restype = vp
        L.rfo_create.argtypes = [i32, i64, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, f64, C.c_uint64, vp]
        L.rfo_destroy.argtypes = [vp]
        L.rfo_round.restype = i32
        L.rfo_round.argtypes = [vp, vp, vp, vp, vp, vp, f64]
        L.rfo_get_state.argtypes = [vp] * 7
        L.rfo_get_edge.argtypes = [vp, i32, vp, vp]
        L.rfo_threads.restype = i32
        L.rfo_set_threads.argtypes = [i32]
        _lib = L
        global _default_threads
        _default_threads = L.rfo_threads()   # OMP_NUM_THREADS, else the visible cores
    return _lib


_default_threads = None


def default_threads():
    _load()
    return _default_threads


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class COracle:
    """R, Cg: CSR graphs (rowptr, col, w in fp64; row = receiver, diagonal included)."""

    def __init__(self, n, p, R, Cg, D, burst, h, c, noise_std=0.0, noise_seed=0, x0=None, threads=None):
        L = _load()
        if threads is not None:
            L.rfo_set_threads(int(threads))
        self.n, self.p = int(n), int(p)
        arrs = [np.ascontiguousarray(R.rowptr, np.int32), np.ascontiguousarray(R.col, np.int32),
                np.ascontiguousarray(R.w, np.float64), np.ascontiguousarray(Cg.rowptr, np.int32),
                np.ascontiguousarray(Cg.col, np.int32), np.ascontiguousarray(Cg.w, np.float64)]
        h = np.ascontiguousarray(h, np.float64).reshape(n, p)
        c = np.ascontiguousarray(c, np.float64).reshape(n, p)
        x0 = None if x0 is None else np.ascontiguousarray(x0, np.float64).reshape(n, p)
        self.eR = int(arrs[0][n]) - n
        self.eC = int(arrs[3][n]) - n
        self.h = L.rfo_create(n, p, *[_p(a) for a in arrs], D, burst, _p(h), _p(c), float(noise_std), int(noise_seed),
                              _p(x0))
        self.threads = L.rfo_threads()

    def round(self, active, delay_R, delay_C, drop_R, drop_C, gamma):
        a = [np.ascontiguousarray(active, np.uint8), np.ascontiguousarray(delay_R, np.int32),
             np.ascontiguousarray(delay_C, np.int32), np.ascontiguousarray(drop_R, np.uint8),
             np.ascontiguousarray(drop_C, np.uint8)]
        if _load().rfo_round(self.h, *[_p(q) for q in a], float(gamma)) != 0:
            raise ValueError("delay outside [0, d_max]")

    def state(self):
        n, p = self.n, self.p
        out = {"x": np.empty((n, p)), "z": np.empty((n, p)), "g": np.empty((n, p)), "t": np.empty(n, np.int64),
               "tau_v": np.empty(max(self.eR, 1), np.int64), "tau_rho": np.empty(max(self.eC, 1), np.int64)}
        _load().rfo_get_state(self.h, *[_p(out[k]) for k in ("x", "z", "g", "t", "tau_v", "tau_rho")])
        out["tau_v"], out["tau_rho"] = out["tau_v"][:self.eR], out["tau_rho"][:self.eC]
        return out

    def edge(self, e):
        rho, rt = np.empty(self.p), np.empty(self.p)
        _load().rfo_get_edge(self.h, int(e), _p(rho), _p(rt))
        return rho, rt

    def close(self):
        if self.h is not None:
            _load().rfo_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
