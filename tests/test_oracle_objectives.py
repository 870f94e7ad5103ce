"""Pins of the oracle's objectives and of its counter-based Gaussian noise."""
import os

import numpy as np
import pytest
import torch

from oracle import objectives as ob

HERE = os.path.dirname(os.path.abspath(__file__))


def test_philox_known_answers():
    with open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        w = [np.array([int(t, 16)], dtype=np.uint64) for t in row]
        out = ob.philox4x32_10(w[0], w[1], w[2], w[3], int(w[4][0]), int(w[5][0]))
        assert [int(o[0]) for o in out] == [int(t[0]) for t in w[6:10]]


def test_gaussian_noise_is_box_muller_of_the_words():
    """Invert Box-Muller: each pair gives back u and the angle of its words."""
    p = 4096
    g = ob.gaussian_noise(5, 3, 9, p).reshape(-1, 4)
    q = np.arange(p // 4, dtype=np.uint64)
    o = ob.philox4x32_10(q, np.zeros_like(q), np.full_like(q, 3), np.full_like(q, 9), 5, 0)
    for a in range(2):
        n0, n1 = g[:, 2 * a], g[:, 2 * a + 1]
        u = np.exp(-(n0 ** 2 + n1 ** 2) / 2)
        np.testing.assert_allclose(u * 2 ** 24, (o[2 * a] >> np.uint64(8)).astype(float) + 1, rtol=1e-9)
        ang = np.mod(np.arctan2(n1, n0), 2 * np.pi)
        ref = 2 * np.pi * o[2 * a + 1].astype(float) / 2 ** 32
        d = np.abs(ang - ref)
        assert np.minimum(d, 2 * np.pi - d).max() < 1e-9


def test_gaussian_noise_moments_and_keys():
    g = ob.gaussian_noise(123, 1, 2, 1 << 20)
    assert abs(g.mean()) < 4e-3 and abs(g.var() - 1) < 6e-3
    assert abs((g ** 3).mean()) < 2e-2 and abs((g ** 4).mean() - 3) < 5e-2
    assert abs(np.corrcoef(g[:-1], g[1:])[0, 1]) < 4e-3
    for other in (ob.gaussian_noise(124, 1, 2, 4096), ob.gaussian_noise(123, 2, 2, 4096),
                  ob.gaussian_noise(123, 1, 3, 4096)):
        assert abs(np.corrcoef(g[:4096], other)[0, 1]) < 0.08
    # prefix property and coordinate subsets
    np.testing.assert_array_equal(ob.gaussian_noise(123, 1, 2, 1001), g[:1001])
    coords = np.array([0, 1, 2, 3, 5, 1000, 77777, (1 << 20) - 1])
    dq = ob.DiagQuadratic(np.ones((2, coords.size)), np.zeros((2, coords.size)), 1.0, 123, coords, 1 << 20)
    np.testing.assert_array_equal(dq.grad(1, np.zeros(coords.size), 2), g[coords])


def _fd(loss, x, eps=1e-6):
    g = np.zeros_like(x)
    for k in range(x.size):
        e = np.zeros_like(x)
        e[k] = eps
        g[k] = (loss(x + e) - loss(x - e)) / (2 * eps)
    return g


def test_gradients_match_finite_differences():
    rng = np.random.default_rng(0)
    n, m, p = 2, 7, 5
    x = rng.standard_normal(p)
    ls = ob.LeastSquares(rng.standard_normal((n, m, p)), rng.standard_normal((n, m)))
    np.testing.assert_allclose(ls.grad(1, x, 0), _fd(lambda v: ls.loss(1, v), x), rtol=1e-6, atol=1e-8)
    lg = ob.Logistic(rng.standard_normal((n, m, p)), (rng.random((n, m)) < 0.5).astype(float), lam=0.3)
    np.testing.assert_allclose(lg.grad(0, x, 0), _fd(lambda v: lg.loss(0, v), x), rtol=1e-6, atol=1e-8)
    dq = ob.DiagQuadratic(rng.uniform(0.5, 2, (n, p)), rng.standard_normal((n, p)))
    np.testing.assert_allclose(dq.grad(1, x, 0), _fd(lambda v: dq.loss(1, v), x), rtol=1e-6, atol=1e-8)
    # minibatch rows = the mean over exactly those rows
    rows = np.array([4, 1, 6])
    sub = ob.Logistic(lg.X[:, rows], lg.y[:, rows], lam=0.3)
    np.testing.assert_allclose(lg.grad(0, x, 3, rows), sub.grad(0, x, 3), rtol=1e-13)
    sub = ob.LeastSquares(ls.A[:, rows], ls.b[:, rows])
    np.testing.assert_allclose(ls.grad(1, x, 3, rows), sub.grad(1, x, 3), rtol=1e-13)


def test_round_bf16_matches_library_conversion():
    rng = np.random.default_rng(1)
    a = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-6, 6, 5000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.005859375, 3.0e38, 1e-40])])
    ref = torch.from_numpy(a).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(ob._round_bf16(a), ref)


def test_softmax_gradient_against_autograd(monkeypatch):
    rng = np.random.default_rng(2)
    n, S, d, K, B = 2, 40, 16, 6, 12
    X = torch.from_numpy(rng.standard_normal((n, S, d))).to(torch.bfloat16).to(torch.float64).numpy()
    lab = rng.integers(0, K, (n, S))
    sm = ob.SoftmaxBf16(X, lab, d, K)
    x = rng.standard_normal(d * K) * 0.5
    rows = rng.choice(S, B, replace=False)

    def autograd(xv):
        W = torch.tensor(xv.reshape(d, K), requires_grad=True)
        loss = torch.nn.functional.cross_entropy(torch.from_numpy(X[1][rows]) @ W, torch.from_numpy(lab[1][rows]))
        loss.backward()
        return W.grad.numpy().reshape(-1)

    # with bf16 rounding: agreement to bf16 accuracy only
    g = sm.grad(1, x, 0, rows)
    ref = autograd(ob._round_bf16(x))
    assert np.linalg.norm(g - ref) / np.linalg.norm(ref) < 4e-3
    # with the rounding switched off: the formula itself, to fp64 accuracy
    monkeypatch.setattr(ob, "_round_bf16", lambda a: np.asarray(a, dtype=np.float64))
    np.testing.assert_allclose(sm.grad(1, x, 0, rows), autograd(x), rtol=1e-10, atol=1e-13)
    # loss = mean cross-entropy over the pool
    W = torch.from_numpy(x.reshape(d, K))
    ref_loss = torch.nn.functional.cross_entropy(torch.from_numpy(X[0]) @ W, torch.from_numpy(lab[0])).item()
    assert abs(sm.loss(0, x) - ref_loss) < 1e-12


def test_logistic_limit_is_the_newton_optimum():
    """No closed form, but the regularised logistic objective is strongly convex: its minimiser is
    found independently by Newton's method on F = sum_i f_i (written out here with the logistic
    Hessian), and the oracle, run with full local gradients over an exponential graph with
    delays and losses, must converge to it although every shard is label-skewed."""
    from oracle.rfast_oracle import RFastOracle
    from rfast_workloads import graphs
    from rfast_workloads.schedule import ScheduleSpec
    n, p, m, lam = 8, 5, 30, 0.3
    rng = np.random.default_rng(12)
    X = rng.standard_normal((n, m, p))
    teacher = rng.standard_normal(p)
    y = (np.einsum("imp,p->im", X, teacher) + 0.5 * rng.standard_normal((n, m)) + 0.8 * (np.arange(n)[:, None] % 2) > 0)
    y = y.astype(np.float64)
    x = np.zeros(p)
    for _ in range(40):                                   # Newton on F
        g, H = np.zeros(p), np.zeros((p, p))
        for i in range(n):
            s = 1.0 / (1.0 + np.exp(-(X[i] @ x)))
            g += X[i].T @ (s - y[i]) / m + lam * x
            H += (X[i].T * (s * (1 - s))) @ X[i] / m + lam * np.eye(p)
        x = x - np.linalg.solve(H, g)
    assert np.abs(g).max() < 1e-13
    x_star = x
    wr, wc = graphs.exponential(n)
    R, C = graphs.from_dense(wr, fp32_weights=False), graphs.from_dense(wc, fp32_weights=False)
    obj = ob.Logistic(X, y, lam)
    local_gap = max(np.abs(obj.grad(i, x_star, 0)).max() for i in range(n))
    assert local_gap > 0.05                               # x* is no node's own optimum
    orc = RFastOracle(n, p, R, C, D=7, burst=4, objective=obj)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, np.full(n, 0.6), 4, 0.15, seed=2)
    for r in range(6000):
        q = sched.round(r)
        orc.round(q.active, q.delay_R, q.delay_C, q.drop_R, q.drop_C, 0.5)
    assert np.abs(orc.x - x_star).max() < 1e-8, np.abs(orc.x - x_star).max()
    assert np.abs(orc.z).max() < 1e-8
