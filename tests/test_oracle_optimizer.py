"""Pins of the labelled optimizer variant (momentum buffer on the tracked
direction, weight decay inside the sampled gradient, step-decayed learning
rate; hyper-parameters of the paper's large-scale experiment).  The paper does
not place them inside Algorithm 1, so the variant is pinned by what the
mathematics fixes: the one-node case is textbook SGD (checked against
torch.optim.SGD + StepLR), the limit point is the minimiser of the decayed
objective, the tracking identity of Lemma 3 is untouched, and beta = lambda = 0
is the paper's method bit for bit.  CPU only."""
import numpy as np
import pytest
import torch

from oracle.objectives import DiagQuadratic, LeastSquares
from oracle.push_pull import PushPullOracle
from oracle.rfast_oracle import RFastOracle, step_gamma
from rfast_workloads import graphs
from rfast_workloads.schedule import ScheduleSpec


def _single_node_graph():
    return graphs.from_dense(np.ones((1, 1)), fp32_weights=False)


def _round_all(orc, gamma, batch=None):
    n = orc.n
    eR, eC = len(orc.edges_R), len(orc.edges_C)
    orc.round(np.ones(n, np.uint8), np.zeros(eR, np.int32), np.zeros(eC, np.int32), np.zeros(eR, np.uint8),
              np.zeros(eC, np.uint8), gamma, batch)


@pytest.mark.parametrize("beta,lam", [(0.9, 1e-2), (0.0, 0.3), (0.6, 0.0)])
def test_one_node_is_textbook_sgd(beta, lam):
    """n = 1 (R = C = [1], no edges): z = g after every step, so the variant is
    x <- x - gamma_r (beta m + g), g = grad f(x) + lambda x: torch's SGD with
    momentum, weight decay and a StepLR schedule."""
    rng = np.random.default_rng(5)
    m, p = 12, 5
    A = rng.standard_normal((1, m, p))
    b = rng.standard_normal((1, m))
    x0 = rng.standard_normal((1, p))
    G = _single_node_graph()
    orc = RFastOracle(1, p, G, G, D=0, burst=1, objective=LeastSquares(A, b), x0=x0, momentum=beta, weight_decay=lam)
    w = torch.tensor(x0[0], dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([w], lr=0.05, momentum=beta, weight_decay=lam)
    sch = torch.optim.lr_scheduler.StepLR(opt, step_size=7, gamma=0.5)
    At, bt = torch.tensor(A[0]), torch.tensor(b[0])
    for r in range(30):
        opt.zero_grad()
        (0.5 / m * ((At @ w - bt) ** 2).sum()).backward()
        opt.step()
        sch.step()
        _round_all(orc, step_gamma(0.05, 0.5, 7, r))
        np.testing.assert_allclose(orc.x[0], w.detach().numpy(), rtol=1e-11, atol=1e-12)


def test_step_gamma_values():
    assert step_gamma(0.1, 0.1, 30, 29) == 0.1
    assert step_gamma(0.1, 0.1, 30, 30) == pytest.approx(0.01)
    assert step_gamma(0.1, 0.1, 30, 89) == pytest.approx(0.001)
    assert step_gamma(0.1, 0.1, 0, 500) == 0.1


def _quadratic(n, p, seed):
    rng = np.random.default_rng(seed)
    h = rng.uniform(0.5, 2.0, (n, p))
    c = rng.standard_normal((n, p)) + np.arange(n)[:, None] / n
    return h, c


@pytest.mark.parametrize("beta", [0.0, 0.5])
def test_limit_is_minimiser_of_decayed_objective(beta):
    """sum_i [f_i(x) + lambda/2 x^2] with f_i = h_i/2 (x - c_i)^2 is minimised at
    sum h_i c_i / (sum h_i + n lambda); asynchrony, delays and losses do not move it."""
    n, p, lam = 8, 4, 0.25
    h, c = _quadratic(n, p, 11)
    wr, wc = graphs.bidirectional_ring(n)
    R, C = graphs.from_dense(wr, fp32_weights=False), graphs.from_dense(wc, fp32_weights=False)
    orc = RFastOracle(n, p, R, C, D=5, burst=3, objective=DiagQuadratic(h, c), momentum=beta, weight_decay=lam)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, p_active=np.full(n, 0.6), d_max=3, p_drop=0.1, seed=3)
    for r in range(6000):
        s = sched.round(r)
        orc.round(s.active, s.delay_R, s.delay_C, s.drop_R, s.drop_C, 0.1 * (1.0 - beta))
    x_star = (h * c).sum(0) / (h.sum(0) + n * lam)
    np.testing.assert_allclose(orc.x, np.broadcast_to(x_star, (n, p)), rtol=0, atol=1e-9)
    plain = (h * c).sum(0) / h.sum(0)
    assert np.abs(plain - x_star).max() > 1e-2      # the decay term really moved the optimum


def test_tracking_identity_and_untouched_buffers():
    """Lemma 3 holds for any gradient sequence, hence also with weight decay inside
    g and with momentum in S1; a node that is not activated keeps x, z, g AND m."""
    n, p = 7, 3
    rng = np.random.default_rng(4)
    wr, wc = graphs.random_digraph(n, rng)
    R, C = graphs.from_dense(wr, fp32_weights=False), graphs.from_dense(wc, fp32_weights=False)
    h, c = _quadratic(n, p, 1)
    orc = RFastOracle(n, p, R, C, D=6, burst=3, objective=DiagQuadratic(h, c, noise_std=0.3, noise_seed=9),
                      x0=rng.standard_normal((n, p)), momentum=0.8, weight_decay=0.05)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, p_active=np.full(n, 0.5), d_max=4, p_drop=0.2, seed=8)
    for r in range(300):
        s = sched.round(r)
        before = (orc.x.copy(), orc.z.copy(), orc.g.copy(), orc.m.copy())
        orc.round(s.active, s.delay_R, s.delay_C, s.drop_R, s.drop_C, 0.02)
        idle = ~s.active.astype(bool)
        for old, new in zip(before, (orc.x, orc.z, orc.g, orc.m)):
            assert np.array_equal(old[idle], new[idle])
        assert np.abs(orc.conservation_residual()).max() < 1e-10 * max(1.0, np.abs(orc.g).max())
    # the stored sample is the decayed one: g_i - lambda x_i - h_i (x_i - c_i) is pure noise of std 0.3
    resid = orc.g - 0.05 * orc.x - h * (orc.x - c)
    assert 0.05 < resid.std() < 0.6


def test_zero_hyperparameters_are_the_plain_method():
    n, p = 6, 4
    rng = np.random.default_rng(0)
    wr, wc = graphs.random_digraph(n, rng)
    R, C = graphs.from_dense(wr), graphs.from_dense(wc)
    h, c = _quadratic(n, p, 2)
    a = RFastOracle(n, p, R, C, D=5, burst=2, objective=DiagQuadratic(h, c))
    b = RFastOracle(n, p, R, C, D=5, burst=2, objective=DiagQuadratic(h, c), momentum=0.0, weight_decay=0.0)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, p_active=np.full(n, 0.5), d_max=4, p_drop=0.1, seed=1)
    for r in range(100):
        s = sched.round(r)
        for o in (a, b):
            o.round(s.active, s.delay_R, s.delay_C, s.drop_R, s.drop_C, 0.05)
    assert np.array_equal(a.x, b.x) and np.array_equal(a.z, b.z)


def test_momentum_first_steps_by_hand():
    """Two nodes, exact small numbers: checks that the buffer starts at zero, takes z
    (not g, not gamma z) and is applied to the node's own descent only."""
    W = np.array([[0.5, 0.5], [0.5, 0.5]])
    R, C = graphs.from_dense(W, fp32_weights=False), graphs.from_dense(W, fp32_weights=False)
    h = np.array([[1.0], [2.0]])
    c = np.array([[1.0], [-1.0]])
    orc = RFastOracle(2, 1, R, C, D=1, burst=1, objective=DiagQuadratic(h, c), momentum=0.5, weight_decay=0.0)
    # x0 = 0: g = z = (-1, 2); round 1: m = z, v = -gamma m = (0.25, -0.5); neighbours' v of version 0 are 0
    _round_all(orc, 0.25)
    np.testing.assert_allclose(orc.m[:, 0], [-1.0, 2.0], atol=0)
    np.testing.assert_allclose(orc.x[:, 0], [0.125, -0.25], atol=1e-15)
    # g' = (1*(0.125-1), 2*(-0.25+1)) = (-0.875, 1.5); z_half = z + g' - g = (-0.875, 1.5); z = z_half / 2
    np.testing.assert_allclose(orc.z[:, 0], [-0.4375, 0.75], atol=1e-15)
    # round 2: m = 0.5 m + z = (-0.9375, 1.75); v = x - 0.25 m = (0.359375, -0.6875); x = (v_i + v_j^1)/2
    _round_all(orc, 0.25)
    np.testing.assert_allclose(orc.m[:, 0], [-0.9375, 1.75], atol=1e-15)
    np.testing.assert_allclose(orc.x[:, 0], [(0.359375 - 0.5) / 2, (-0.6875 + 0.25) / 2], atol=1e-15)


def test_push_pull_variant_matches_centralised_heavy_ball():
    """W = A = 11^T/n and identical quadratics: every node holds the same x, z is the
    common gradient, and eq. (2) with the variant is heavy-ball gradient descent on
    f + lambda/2 x^2, whose iterates are written out directly."""
    n, p, beta, lam, gamma = 4, 3, 0.7, 0.1, 0.2
    rng = np.random.default_rng(6)
    h1, c1 = rng.uniform(0.5, 2.0, p), rng.standard_normal(p)
    h, c = np.tile(h1, (n, 1)), np.tile(c1, (n, 1))
    J = np.full((n, n), 1.0 / n)
    x0 = np.tile(rng.standard_normal(p), (n, 1))
    pp = PushPullOracle(J, J, DiagQuadratic(h, c), x0=x0, momentum=beta, weight_decay=lam)
    x, m = x0[0].copy(), np.zeros(p)
    for _ in range(50):
        m = beta * m + h1 * (x - c1) + lam * x
        x = x - gamma * m
        pp.step(gamma)
        np.testing.assert_allclose(pp.x, np.tile(x, (n, 1)), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(x, h1 * c1 / (h1 + lam), atol=1e-3)
