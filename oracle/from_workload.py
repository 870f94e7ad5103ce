"""Builds the fp64 oracle for a Workload of rfast_workloads (test infrastructure, like the rest
of oracle/: only the tests, the smoke check and the CPU-baseline leg of the benchmark call it)."""
from __future__ import annotations

from . import objectives as ob
from .rfast_oracle import RFastOracle


def make_oracle(w, coords=None, x0=None, momentum=0.0, weight_decay=0.0):
    """coords: run the separable objective on this subset of coordinates only (the noise counters
    keep indexing the full vector, so those coordinates evolve exactly as inside it)."""
    d = w.data
    p = w.p
    if w.objective == "diag_quadratic":
        if coords is None:
            obj = ob.DiagQuadratic(d["h"], d["c"], w.noise_std, w.noise_seed)
        else:
            obj = ob.DiagQuadratic(d["h"][:, coords], d["c"][:, coords], w.noise_std, w.noise_seed, coords, w.p)
            p = len(coords)
    elif w.objective == "least_squares":
        obj = ob.LeastSquares(d["A"], d["b"])
    elif w.objective == "logistic":
        obj = ob.Logistic(d["X"], d["y"])
    else:
        from rfast_workloads.problems import bf16_bits_to_f32
        obj = ob.SoftmaxBf16(bf16_bits_to_f32(d["Xb"]), d["labels"], w.extra["d"], w.extra["K"])
    b0 = w.sched.initial_batch()
    return RFastOracle(w.n, p, w.R, w.C, w.D, w.burst, obj, x0=x0, batch0=b0, momentum=momentum,
                       weight_decay=weight_decay)
