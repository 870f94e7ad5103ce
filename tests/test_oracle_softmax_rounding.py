"""How far the bf16 reading of config 4 sits from problem (1)'s own gradient.

The oracle of the softmax workload (oracle.objectives.SoftmaxBf16) rounds W and E = (P - Y)/B to bf16 where
the kernel does, because the workload asks for bf16 GEMM inputs.  That makes the oracle's structure follow the
kernel's at exactly those two points, so it is pinned here against the definition with no rounding at all:
the gradient of the mean cross-entropy of softmax regression, written out below in fp64.  The sampled
gradient of Assumption 5 must be unbiased; rounding perturbs it by a relative 2^-9 per operand entry, and the
tests below bound what that does to a gradient and to a whole trajectory."""
import numpy as np

from oracle.objectives import SoftmaxBf16
from oracle.rfast_oracle import RFastOracle
from rfast_workloads import configs
from rfast_workloads.problems import bf16_bits_to_f32


class PlainSoftmax:
    """grad of (1/B) sum_s [logsumexp(W^T a_s) - (W^T a_s)[y_s]] in fp64, nothing rounded."""

    def __init__(self, X_pool, labels, d, K):
        self.X, self.lab, self.d, self.K = np.asarray(X_pool, np.float64), np.asarray(labels, np.int64), d, K
        self.p = d * K

    def grad(self, i, x, version, batch=None):
        rows = np.arange(self.X.shape[1]) if batch is None else np.asarray(batch)
        A, y = self.X[i][rows], self.lab[i][rows]
        logits = A @ x.reshape(self.d, self.K)
        P = np.exp(logits - np.logaddexp.reduce(logits, axis=1, keepdims=True))
        P[np.arange(len(rows)), y] -= 1.0
        return (A.T @ P / len(rows)).reshape(-1)


def _small():
    return configs.config4(d=64, K=32, samples=256, batch=64, rounds=300)


def test_rounded_gradient_is_close_to_the_definition():
    w = _small()
    X = bf16_bits_to_f32(w.data["Xb"])
    a, b = SoftmaxBf16(X, w.data["labels"], 64, 32), PlainSoftmax(X, w.data["labels"], 64, 32)
    rng = np.random.default_rng(5)
    worst = 0.0
    for trial in range(20):
        x = rng.standard_normal(w.p) * (0.02 if trial % 2 else 1.0)
        rows = rng.choice(256, size=64, replace=False)
        ga, gb = a.grad(trial % w.n, x, 0, rows), b.grad(trial % w.n, x, 0, rows)
        worst = max(worst, float(np.linalg.norm(ga - gb) / np.linalg.norm(gb)))
    print("worst relative distance of the bf16-rounded gradient from the fp64 definition:", worst)
    # two operands rounded to 8 significant bits each: errors of relative size 2^-9, largely independent
    assert worst <= 2.0 ** -7


def test_rounded_trajectory_stays_near_the_unrounded_one():
    w = _small()
    X = bf16_bits_to_f32(w.data["Xb"])
    b0 = w.sched.initial_batch()
    runs = [RFastOracle(w.n, w.p, w.R, w.C, w.D, w.burst, obj(X, w.data["labels"], 64, 32), batch0=b0)
            for obj in (SoftmaxBf16, PlainSoftmax)]
    worst_x = worst_z = 0.0
    for r in range(300):
        q = w.sched.round(r)
        for o in runs:
            o.round(q.active, q.delay_R, q.delay_C, q.drop_R, q.drop_C, w.gamma, q.batch_idx)
        if (r + 1) % 100 == 0:
            a, b = runs
            dx = float(np.linalg.norm(a.x - b.x) / np.linalg.norm(b.x))
            dz = float(np.linalg.norm(a.z - b.z) / max(np.linalg.norm(b.z), 1e-3 * np.linalg.norm(b.g)))
            worst_x, worst_z = max(worst_x, dx), max(worst_z, dz)
            print(f"round {r + 1}: rounded vs unrounded oracle, rel-L2 x {dx:.2e} z {dz:.2e}")
            assert np.array_equal(a.t, b.t)
    # the distance between the two readings, next to the 2e-3 the GPU is held to against the rounded one
    assert worst_x <= 5e-3 and worst_z <= 2e-2
