"""TEST INFRASTRUCTURE — fp64 local objectives f_i and their stochastic
gradients for the oracle (problem (1) of the paper: F = sum_i f_i, each node
samples an unbiased gradient of its own f_i, Assumption 5).

Only tests, the smoke check and the benchmark's cpu_baseline leg import this.
No code is shared with the HIP library; the counter-based generator below is
implemented here on its own from its published definition.

Each objective offers  grad(i, x, version, batch_rows) -> float64 [p]  (the
sample is identified by the node's local iteration stamp `version`, 0 for the
initial gradient) and  loss(i, x) -> float  (the full local loss).

Pins (tests/test_oracle_objectives.py, tests/test_oracle_pins.py): every gradient against
finite differences of its loss; the softmax gradient against autograd and its bf16
rounding against the library conversion; the generator against published known-answer
vectors; the limits of least-squares, diagonal-quadratic and logistic runs against the
closed-form / Newton optimum.  Parity unpinned: the limit of runs with SoftmaxBf16 (the
bf16 rounding of W makes its gradient piecewise constant: no exact limit point exists).
"""
from __future__ import annotations

import numpy as np

# ---------------------------------------------------------------- Philox4x32-10
# Counter-based generator of Salmon, Moraes, Dror and Shaw, "Parallel random
# numbers: as easy as 1, 2, 3" (SC'11): ten rounds of two 32x32->64 multiplies
# on a 4-word counter with a 2-word key bumped by Weyl constants.
_PH_M0 = np.uint64(0xD2511F53)
_PH_M1 = np.uint64(0xCD9E8D57)
_PH_W0 = np.uint64(0x9E3779B9)
_PH_W1 = np.uint64(0xBB67AE85)
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Vectorised over equal-shaped uint64 arrays holding 32-bit words."""
    c0, c1, c2, c3 = (np.asarray(a, dtype=np.uint64) & _MASK for a in (c0, c1, c2, c3))
    k0 = np.uint64(k0) & _MASK
    k1 = np.uint64(k1) & _MASK
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + _PH_W0) & _MASK
            k1 = (k1 + _PH_W1) & _MASK
        p0 = _PH_M0 * c0
        p1 = _PH_M1 * c2
        hi0, lo0 = p0 >> _S32, p0 & _MASK
        hi1, lo1 = p1 >> _S32, p1 & _MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return c0, c1, c2, c3


def gaussian_noise(seed, node, version, p):
    """Standard normals for coordinates 0..p-1 of (node, version).

    Integer stage (must match the kernel bit for bit): coordinates are taken in
    groups of four; group q uses counter (q mod 2^32, q div 2^32, node, version)
    under key (seed mod 2^32, seed div 2^32) and yields words o0..o3.
    Float stage (Box-Muller): u = ((o >> 8) + 1) / 2^24 in (0, 1],
    angle = 2*pi*o' / 2^32; (o0, o1) gives coordinates 4q, 4q+1 as
    r*cos, r*sin with r = sqrt(-2 ln u); (o2, o3) gives 4q+2, 4q+3."""
    q = np.arange((p + 3) // 4, dtype=np.uint64)
    o0, o1, o2, o3 = philox4x32_10(q & _MASK, q >> _S32, np.full_like(q, node), np.full_like(q, version),
                                   int(seed) & 0xFFFFFFFF, (int(seed) >> 32) & 0xFFFFFFFF)
    out = np.empty((q.shape[0], 4), dtype=np.float64)
    for a, (ou, oa) in enumerate(((o0, o1), (o2, o3))):
        u = ((ou >> np.uint64(8)).astype(np.float64) + 1.0) / 16777216.0
        ang = (2.0 * np.pi) * (oa.astype(np.float64) / 4294967296.0)
        r = np.sqrt(-2.0 * np.log(u))
        out[:, 2 * a] = r * np.cos(ang)
        out[:, 2 * a + 1] = r * np.sin(ang)
    return out.reshape(-1)[:p]


# ------------------------------------------------------------------ objectives
class DiagQuadratic:
    """f_i(x) = 1/2 sum_k h_ik (x_k - c_ik)^2; sampled gradient = h*(x - c) +
    noise_std * N(0, I), the noise keyed by (seed, node, version, coordinate).
    `coords` restricts the oracle to a subset of coordinates (the objective is
    separable, so a subset evolves exactly as it does inside the full vector)."""

    def __init__(self, h, c, noise_std=0.0, noise_seed=0, coords=None, p_full=None):
        self.h = np.asarray(h, dtype=np.float64)
        self.c = np.asarray(c, dtype=np.float64)
        self.noise_std, self.noise_seed = float(noise_std), int(noise_seed)
        self.coords = None if coords is None else np.asarray(coords, dtype=np.int64)
        self.p_full = self.h.shape[1] if p_full is None else int(p_full)
        self.p = self.h.shape[1]

    def grad(self, i, x, version, batch=None):
        g = self.h[i] * (x - self.c[i])
        if self.noise_std != 0.0:
            if self.coords is None:
                g = g + self.noise_std * gaussian_noise(self.noise_seed, i, version, self.p_full)
            else:
                g = g + self.noise_std * self._noise_at(i, version)
        return g

    def _noise_at(self, i, version):
        k = self.coords.astype(np.uint64)
        q = k >> np.uint64(2)
        o = philox4x32_10(q & _MASK, q >> _S32, np.full_like(q, i), np.full_like(q, version),
                          self.noise_seed & 0xFFFFFFFF, (self.noise_seed >> 32) & 0xFFFFFFFF)
        lane = (k & np.uint64(3)).astype(np.int64)
        ou = np.where(lane < 2, o[0], o[2])
        oa = np.where(lane < 2, o[1], o[3])
        u = ((ou >> np.uint64(8)).astype(np.float64) + 1.0) / 16777216.0
        ang = (2.0 * np.pi) * (oa.astype(np.float64) / 4294967296.0)
        r = np.sqrt(-2.0 * np.log(u))
        return np.where(lane % 2 == 0, r * np.cos(ang), r * np.sin(ang))

    def loss(self, i, x):
        return float(0.5 * np.sum(self.h[i] * (x - self.c[i]) ** 2))


class LeastSquares:
    """f_i(x) = (1/2m) ||A_i x - b_i||^2; batch rows None = all m rows."""

    def __init__(self, A, b):
        self.A = np.asarray(A, dtype=np.float64)
        self.b = np.asarray(b, dtype=np.float64)
        self.p = self.A.shape[2]

    def grad(self, i, x, version, batch=None):
        A, b = (self.A[i], self.b[i]) if batch is None else (self.A[i][batch], self.b[i][batch])
        return A.T @ (A @ x - b) / A.shape[0]

    def loss(self, i, x):
        r = self.A[i] @ x - self.b[i]
        return float(r @ r / (2.0 * self.A.shape[1]))


class Logistic:
    """f_i(x) = mean_s [ log(1 + exp(a_s.x)) - y_s a_s.x ] + lam/2 ||x||^2, labels in {0, 1}."""

    def __init__(self, X, y, lam=0.0):
        self.X = np.asarray(X, dtype=np.float64)
        self.y = np.asarray(y, dtype=np.float64)
        self.lam = float(lam)
        self.p = self.X.shape[2]

    def grad(self, i, x, version, batch=None):
        X, y = (self.X[i], self.y[i]) if batch is None else (self.X[i][batch], self.y[i][batch])
        s = 1.0 / (1.0 + np.exp(-(X @ x)))
        return X.T @ (s - y) / X.shape[0] + self.lam * x

    def loss(self, i, x):
        m = self.X[i] @ x
        return float(np.mean(np.logaddexp(0.0, m) - self.y[i] * m) + 0.5 * self.lam * (x @ x))


def _round_bf16(a):
    """fp64 -> fp32 (round to nearest even) -> bf16 (round to nearest even),
    returned as float64 holding the bf16 value: the precision in which the
    kernel takes the same rounding decision."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)
    return (u.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


class SoftmaxBf16:
    """Softmax regression on a minibatch with bf16 GEMM inputs and wide
    accumulation: x is W (d x K, row-major: W[f, k] = x[f*K + k]);
    logits = Xb @ bf16(W); P = softmax(logits) row-wise;
    E = bf16((P - onehot) / B); grad = Xb^T @ E.
    f_i = mean cross-entropy over the node's pool (evaluated with the same
    rounded W)."""

    def __init__(self, X_pool, labels, d, K):
        self.X = np.asarray(X_pool, dtype=np.float64)       # [n, samples, d], bf16-representable
        self.lab = np.asarray(labels, dtype=np.int64)
        self.d, self.K = int(d), int(K)
        self.p = self.d * self.K

    def grad(self, i, x, version, batch=None):
        rows = np.arange(self.X.shape[1]) if batch is None else np.asarray(batch)
        Xb = self.X[i][rows]
        Wq = _round_bf16(x.reshape(self.d, self.K))
        logits = Xb @ Wq
        logits = logits - logits.max(axis=1, keepdims=True)
        P = np.exp(logits)
        P /= P.sum(axis=1, keepdims=True)
        P[np.arange(rows.shape[0]), self.lab[i][rows]] -= 1.0
        E = _round_bf16(P / rows.shape[0])
        return (Xb.T @ E).reshape(-1)

    def loss(self, i, x):
        Wq = _round_bf16(x.reshape(self.d, self.K))
        logits = self.X[i] @ Wq
        lse = np.logaddexp.reduce(logits, axis=1)
        return float(np.mean(lse - logits[np.arange(logits.shape[0]), self.lab[i]]))
