"""Pins of the synchronous push-pull oracle (eq. (2) of the paper)."""
import numpy as np

from oracle.objectives import DiagQuadratic, LeastSquares
from oracle.push_pull import PushPullOracle
from rfast_workloads import graphs


def test_complete_averaging_reduces_to_gradient_descent():
    """With W = A = (1/n) 1 1^T every node holds xbar after one step and
    xbar^{t+1} = xbar^t - gamma * (1/n) sum_i grad f_i(xbar^t) from then on: for the
    diagonal quadratic, coordinate-wise xbar^{t+1} - x* = (1 - gamma*mean_i h_i)(xbar^t - x*)."""
    n, p, gamma = 5, 7, 0.3
    rng = np.random.default_rng(0)
    h, c = rng.uniform(0.5, 2, (n, p)), rng.standard_normal((n, p))
    J = np.full((n, n), 1.0 / n)
    orc = PushPullOracle(J, J, DiagQuadratic(h, c), x0=rng.standard_normal((n, p)))
    x_star = (h * c).sum(0) / h.sum(0)
    orc.step(gamma)
    assert np.abs(orc.x - orc.x.mean(0)).max() < 1e-15
    # tracker conservation: 1^T z = 1^T grad f(x) (A is column-stochastic)
    np.testing.assert_allclose(orc.z.sum(0), orc.g.sum(0), atol=1e-13)
    # from step 1 on z_i = mean gradient at the common point... after one more step
    orc.step(gamma)
    e_prev = orc.x[0] - x_star
    for _ in range(20):
        orc.step(gamma)
        e = orc.x[0] - x_star
        np.testing.assert_allclose(e, (1 - gamma * h.mean(0)) * e_prev, rtol=1e-9, atol=1e-15)
        np.testing.assert_allclose(orc.z.sum(0), orc.g.sum(0), atol=1e-12)
        e_prev = e


def test_converges_to_global_optimum_over_spanning_trees():
    """Push-pull needs only spanning trees with a common root (Assumption 2)."""
    n, p = 8, 4
    rng = np.random.default_rng(1)
    A_ = rng.standard_normal((n, 9, p))
    b_ = rng.standard_normal((n, 9))
    x_star = np.linalg.solve(sum(A_[i].T @ A_[i] for i in range(n)), sum(A_[i].T @ b_[i] for i in range(n)))
    for build, gamma in ((graphs.tree_pull_star_push, 0.02), (graphs.directed_ring, 0.04)):
        W, A = build(n)
        orc = PushPullOracle(W, A, LeastSquares(A_, b_))
        for _ in range(12000):
            orc.step(gamma)
        assert np.abs(orc.x - x_star).max() < 1e-9
        assert np.abs(orc.z).max() < 1e-9
