"""The five synthetic workloads, restated as data.

Each stands in for a workload of the paper that cannot be present here:
config 1 takes the structure of the paper's logistic-regression experiment
(binary labels, heterogeneous shards), config 2 the flat-vector size of its
image-classification model, config 3 the structure of its straggler
experiment over a parameter-server-like pair of spanning trees.  Sizes can be
shrunk (`p`, `samples`, `rounds`) for parity cases the oracle finishes in
seconds; graph, schedule law and value distributions stay the same.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from . import graphs, problems
from .schedule import ScheduleSpec, straggler_probs

BURST = 4  # a version is force-delivered once the BURST-1 before it were all lost


@dataclass
class Workload:
    name: str
    n: int
    p: int
    R: graphs.CSRGraph
    C: graphs.CSRGraph
    D: int                 # maximum staleness in sender versions; ring has D+2 slots
    burst: int
    gamma: float
    rounds: int
    objective: str         # "least_squares" | "logistic" | "diag_quadratic" | "softmax_bf16"
    data: dict
    sched: ScheduleSpec
    noise_std: float = 0.0
    noise_seed: int = 0
    tol: float = 1e-4
    extra: dict = field(default_factory=dict)


def _mk(name, n, p, dense_r, dense_c, d_max, gamma, rounds, objective, data, p_active,
        p_drop, seed, batch=0, samples=0, noise_std=0.0, tol=1e-4, burst=BURST, extra=None):
    R = graphs.from_dense(dense_r)
    C = graphs.from_dense(dense_c)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, np.broadcast_to(np.asarray(p_active, float), (n,)).copy(),
                         d_max, p_drop, batch, samples, seed)
    return Workload(name, n, p, R, C, d_max + burst - 1, burst, gamma, rounds, objective, data,
                    sched, noise_std, seed + 12345, tol, extra or {})


def config0(seed=0, rounds=2000, p=64, m=32):
    n = 8
    r, c = graphs.directed_ring(n)
    return _mk("cfg0_ring8_least_squares", n, p, r, c, 3, 0.02, rounds, "least_squares",
               problems.least_squares(n, p, m, seed), 0.5, 0.1, seed, samples=m)


def config1(seed=0, rounds=5000, p=4096, samples=2048, batch=64):
    n = 32
    r, c = graphs.exponential(n)
    return _mk("cfg1_exp32_logistic", n, p, r, c, 8, 0.05, rounds, "logistic",
               problems.logistic(n, p, samples, seed), 0.5, 0.05, seed, batch=batch, samples=samples)


def config2(seed=0, rounds=500, p=11_200_000, gamma=0.05):
    n = 16
    r, c = graphs.bidirectional_ring(n)
    return _mk("cfg2_biring16_diagquad", n, p, r, c, 4, gamma, rounds, "diag_quadratic",
               problems.diag_quadratic(n, p, seed), 1.0, 0.02, seed, noise_std=0.1)


def config3(seed=0, rounds=2000, p=1_048_576, gamma=2e-4):
    n = 64
    r, c = graphs.tree_pull_star_push(n)
    return _mk("cfg3_tree_star64_diagquad", n, p, r, c, 16, gamma, rounds, "diag_quadratic",
               problems.diag_quadratic(n, p, seed), straggler_probs(n, seed), 0.2, seed, noise_std=0.1)


def config4(seed=0, rounds=3000, d=1024, K=128, samples=2048, batch=256):
    n = 128
    r, c = graphs.exponential(n)
    return _mk("cfg4_exp128_softmax_bf16", n, d * K, r, c, 8, 0.1, rounds, "softmax_bf16",
               problems.softmax_pool(n, d, K, samples, seed), 0.5, 0.05, seed,
               batch=batch, samples=samples, tol=2e-3, extra={"d": d, "K": K})


CONFIGS = [config0, config1, config2, config3, config4]
