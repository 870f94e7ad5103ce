"""Puts a Workload on the GPU: the library context for it and device copies of stretches of its
schedule.  Argument marshalling only (the library does the work); imports torch and the binding
lazily, so the generators of this package stay importable without either."""
from __future__ import annotations

import numpy as np


def csr(g):
    return (g.rowptr, g.col, g.w32())


def make_gpu(w, device="cuda:0"):
    """An RFast context (paper_2307_11617_amd.RFast) for workload w, objective data uploaded."""
    import torch
    from paper_2307_11617_amd import RFast
    d = w.data
    if w.objective == "diag_quadratic":
        d0, d1 = torch.from_numpy(d["h"]), torch.from_numpy(d["c"])
        kw = dict(noise_std=w.noise_std, noise_seed=w.noise_seed)
    elif w.objective == "least_squares":
        d0, d1 = torch.from_numpy(d["A"]), torch.from_numpy(d["b"])
        kw = dict(samples=d["A"].shape[1], batch=w.sched.batch)
    elif w.objective == "logistic":
        d0, d1 = torch.from_numpy(d["X"]), torch.from_numpy(d["y"])
        kw = dict(samples=d["X"].shape[1], batch=w.sched.batch)
    else:
        d0 = torch.from_numpy(d["Xb"].view(np.int16)).view(torch.bfloat16)
        d1 = torch.from_numpy(d["labels"])
        kw = dict(samples=d["Xb"].shape[1], batch=w.sched.batch, d=w.extra["d"], K=w.extra["K"])
    return RFast(w.n, w.p, csr(w.R), csr(w.C), w.D, w.burst, w.objective, d0, d1, device=device, **kw)


def upload_chunk(gpu, w, r0, r1):
    """Rounds r0..r1-1 of w's schedule, stacked: (host arrays, device tensors)."""
    import torch
    st = w.sched.stacked(r0, r1)
    dev = {k: (None if v is None else torch.from_numpy(v).to(gpu.device)) for k, v in st.items()}
    return st, dev
