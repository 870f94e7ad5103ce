"""Seeded asynchrony schedules: who is active, how stale each edge is, which
packets are lost, which samples are drawn.

A schedule is pure input to both the oracle and the GPU library (Assumption 3
of the paper describes the admissible ones: every node active within a bounded
window, delays bounded by D).  Round r's draw depends only on (seed, r), so any
round can be produced on its own.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class RoundInputs:
    active: np.ndarray    # uint8 [n]
    delay_R: np.ndarray   # int32 [nnzR_off], rounds, 0..d_max
    delay_C: np.ndarray   # int32 [nnzC_off]
    drop_R: np.ndarray    # uint8 [nnzR_off]: the packet SENT on this edge this round is lost
    drop_C: np.ndarray    # uint8 [nnzC_off]
    batch_idx: np.ndarray | None  # int32 [n, batch] sample rows for this round's gradient


@dataclass
class ScheduleSpec:
    n: int
    nnzR_off: int
    nnzC_off: int
    p_active: np.ndarray  # float64 [n] activation probability per node
    d_max: int
    p_drop: float
    batch: int = 0        # 0: no minibatch indices
    samples: int = 0      # rows per node to draw from
    seed: int = 0

    def _rng(self, r: int) -> np.random.Generator:
        return np.random.Generator(np.random.PCG64(np.random.SeedSequence([self.seed, 77, r + 1])))

    def round(self, r: int) -> RoundInputs:
        g = self._rng(r)
        active = (g.random(self.n) < self.p_active).astype(np.uint8)
        dR = g.integers(0, self.d_max + 1, self.nnzR_off, dtype=np.int32)
        dC = g.integers(0, self.d_max + 1, self.nnzC_off, dtype=np.int32)
        xR = (g.random(self.nnzR_off) < self.p_drop).astype(np.uint8)
        xC = (g.random(self.nnzC_off) < self.p_drop).astype(np.uint8)
        bi = self._batch(g)
        return RoundInputs(active, dR, dC, xR, xC, bi)

    def _batch(self, g: np.random.Generator):
        if self.batch <= 0:
            return None
        out = np.empty((self.n, self.batch), dtype=np.int32)
        for i in range(self.n):
            out[i] = g.choice(self.samples, size=self.batch, replace=False)
        return out

    def initial_batch(self):
        """Sample indices for the initial gradient z^0 = g^0 (Algorithm 1, initialisation)."""
        return self._batch(self._rng(-1))

    def stacked(self, r0: int, r1: int):
        """Rounds r0..r1-1 stacked along a leading axis (device-resident schedules)."""
        rs = [self.round(r) for r in range(r0, r1)]
        out = {
            "active": np.stack([q.active for q in rs]),
            "delay_R": np.stack([q.delay_R for q in rs]),
            "delay_C": np.stack([q.delay_C for q in rs]),
            "drop_R": np.stack([q.drop_R for q in rs]),
            "drop_C": np.stack([q.drop_C for q in rs]),
            "batch_idx": None if self.batch <= 0 else np.stack([q.batch_idx for q in rs]),
        }
        return out


def straggler_probs(n: int, seed: int, frac: float = 0.1, slow: float = 0.05, fast: float = 0.6):
    """floor(frac*n) nodes of a seeded permutation are slow, the others fast."""
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 78])))
    perm = g.permutation(n)
    pr = np.full(n, fast)
    pr[perm[: int(np.floor(frac * n))]] = slow
    return pr
