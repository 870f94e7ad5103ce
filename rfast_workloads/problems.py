"""Seeded synthetic objective data for the five workloads.

Everything here is data preparation only: arrays are drawn in float64, rounded
once to the storage type the GPU library is given (fp32, or bf16 for the
softmax pool) and handed to both sides as those very values.  No gradient,
loss or update rule lives in this module.
"""
from __future__ import annotations

import numpy as np


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, stream])))


def f32(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def to_bf16_bits(a32: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(a32, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def least_squares(n: int, p: int, m: int, seed: int):
    """f_i(x) = (1/2m) ||A_i x - b_i||^2 with A_i ~ N(i/n, 1) entrywise and
    b_i = A_i x_teacher + 0.1 N(0,1): heterogeneous shards, one shared teacher."""
    rng = _rng(seed, 10)
    teacher = rng.standard_normal(p)
    A = np.empty((n, m, p), dtype=np.float32)
    b = np.empty((n, m), dtype=np.float32)
    for i in range(n):
        Ai = f32(rng.standard_normal((m, p)) + i / n)
        A[i] = Ai
        b[i] = f32(Ai.astype(np.float64) @ teacher + 0.1 * rng.standard_normal(m))
    return {"A": A, "b": b, "teacher": teacher}


def logistic(n: int, p: int, samples: int, seed: int, skew: float = 0.75):
    """Binary logistic data: features N(0, 1/p), labels 1[a.w > 0] from one
    random teacher w.  Node i holds round(skew*samples) rows of class i mod 2
    and the rest of the other class (filled by rejection)."""
    rng = _rng(seed, 11)
    w = rng.standard_normal(p)
    X = np.empty((n, samples, p), dtype=np.float32)
    y = np.empty((n, samples), dtype=np.float32)
    n_dom = int(round(skew * samples))
    for i in range(n):
        dom = i % 2
        need = {dom: n_dom, 1 - dom: samples - n_dom}
        rows, labs = [], []
        while need[0] > 0 or need[1] > 0:
            cand = f32(rng.standard_normal((samples, p)) / np.sqrt(p))
            lab = (cand.astype(np.float64) @ w > 0).astype(np.int64)
            for cls in (0, 1):
                if need[cls] > 0:
                    idx = np.nonzero(lab == cls)[0][: need[cls]]
                    rows.append(cand[idx])
                    labs.append(np.full(idx.shape[0], cls, dtype=np.float32))
                    need[cls] -= idx.shape[0]
        Xi = np.concatenate(rows, axis=0)
        yi = np.concatenate(labs, axis=0)
        perm = rng.permutation(samples)
        X[i] = Xi[perm]
        y[i] = yi[perm]
    return {"X": X, "y": y, "teacher": w}


def diag_quadratic(n: int, p: int, seed: int):
    """f_i(x) = 1/2 sum_k h_ik (x_k - c_ik)^2, h ~ U[0.5, 2], c_ik ~ N(i/n, 1)."""
    rng = _rng(seed, 12)
    h = np.empty((n, p), dtype=np.float32)
    c = np.empty((n, p), dtype=np.float32)
    for i in range(n):
        h[i] = rng.uniform(0.5, 2.0, p).astype(np.float32)
        c[i] = (rng.standard_normal(p, dtype=np.float32) + np.float32(i / n))
    return {"h": h, "c": c}


def softmax_pool(n: int, d: int, K: int, samples: int, seed: int, alpha: float = 0.3):
    """Class-conditional Gaussian pool: shared class means mu_y ~ N(0, I)/sqrt(d),
    sample = mu_y + N(0, I/d); node i draws labels from its own Dirichlet(alpha)
    mixture.  Features are rounded to bf16 once; both sides use those values."""
    rng = _rng(seed, 13)
    mu = rng.standard_normal((K, d)) / np.sqrt(d)
    Xb = np.empty((n, samples, d), dtype=np.uint16)
    lab = np.empty((n, samples), dtype=np.int32)
    for i in range(n):
        mix = rng.dirichlet(np.full(K, alpha))
        li = rng.choice(K, size=samples, p=mix).astype(np.int32)
        xi = mu[li] + rng.standard_normal((samples, d)) / np.sqrt(d)
        Xb[i] = to_bf16_bits(f32(xi))
        lab[i] = li
    return {"Xb": Xb, "labels": lab, "mu": mu}
