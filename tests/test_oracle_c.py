"""Pins of the plain-C oracle (oracle/rfast_oracle_c.c): the hand-stepped n = 3
example in exact rationals, Lemma 3, the closed-form limit, and agreement with the
separately written NumPy oracle on random graphs and schedules (stamps bit for
bit, vectors to rounding).  CPU only."""
import numpy as np
import pytest

from oracle.c_oracle import COracle, build_c_oracle
from oracle.objectives import DiagQuadratic
from oracle.rfast_oracle import RFastOracle
from rfast_workloads import graphs
from rfast_workloads.schedule import ScheduleSpec

from test_oracle_pins import _parse_golden


@pytest.fixture(scope="module", autouse=True)
def _built():
    build_c_oracle()


def test_hand_stepped_n3_example_exact():
    """Every value of the golden file is a dyadic rational: fp64 reproduces it exactly."""
    r, c = graphs.directed_ring(3)
    R, C = graphs.from_dense(r), graphs.from_dense(c)
    orc = COracle(3, 1, R, C, 2, 2, np.array([[1.0], [2.0], [1.0]]), np.array([[1.0], [2.0], [4.0]]))
    assert orc.state()["z"][:, 0].tolist() == [-1.0, -4.0, -4.0]
    perm = [1, 2, 0]   # CSR edge ids (0<-2), (1<-0), (2<-1); golden order (1,0), (2,1), (0,2)
    sched = [
        dict(active=[1, 1, 0], dR=[0, 0, 0], dC=[0, 0, 0], xR=[0, 0, 0], xC=[0, 0, 1]),
        dict(active=[0, 1, 1], dR=[0, 1, 0], dC=[0, 1, 0], xR=[0, 0, 0], xC=[0, 0, 0]),
        dict(active=[1, 1, 1], dR=[0, 0, 0], dC=[0, 0, 0], xR=[0, 0, 0], xC=[0, 0, 0]),
    ]
    stamps_after = [([0, 0, 0], [0, 0, 0]), ([0, 0, 1], [0, 0, 0]), ([1, 1, 2], [1, 1, 2])]
    for k, (s, gd) in enumerate(zip(sched, _parse_golden())):
        orc.round(s["active"], s["dR"], s["dC"], s["xR"], s["xC"], 0.25)
        st = orc.state()
        assert st["x"][:, 0].tolist() == gd["x"], k
        assert st["z"][:, 0].tolist() == gd["z"], k
        assert st["g"][:, 0].tolist() == gd["g"], k
        assert st["t"].tolist() == gd["t"], k
        assert (st["tau_v"].tolist(), st["tau_rho"].tolist()) == stamps_after[k], k
        edges = [orc.edge(e) for e in perm]
        assert [e[0][0] for e in edges] == gd["rho"], k
        assert [e[1][0] for e in edges] == gd["rho_t"], k


def _instance(seed, n, p, noise):
    rng = np.random.default_rng(seed)
    wr, wc = graphs.random_digraph(n, rng, extra=0.4)
    R, C = graphs.from_dense(wr), graphs.from_dense(wc)
    h = rng.uniform(0.5, 2.0, (n, p))
    c = rng.standard_normal((n, p))
    x0 = rng.standard_normal((n, p))
    return R, C, h, c, x0


@pytest.mark.parametrize("seed,threads", [(0, 1), (1, 4), (2, 3)])
def test_agrees_with_numpy_oracle(seed, threads):
    """Two implementations written separately from the paper: same stamps, same vectors."""
    n, p, D, burst = [6, 9, 12][seed], [7, 18, 5][seed], [5, 7, 9][seed], [2, 4, 6][seed]
    R, C, h, c, x0 = _instance(seed, n, p, 0.2)
    a = COracle(n, p, R, C, D, burst, h, c, noise_std=0.2, noise_seed=42 + seed, x0=x0, threads=threads)
    b = RFastOracle(n, p, R, C, D, burst, DiagQuadratic(h, c, 0.2, 42 + seed), x0=x0)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, np.full(n, [0.5, 0.3, 0.8][seed]), D - burst + 1, [0.2, 0.5, 0.7][seed],
                         seed=seed)
    for r in range(250):
        q = sched.round(r)
        a.round(q.active, q.delay_R, q.delay_C, q.drop_R, q.drop_C, 0.03)
        b.round(q.active, q.delay_R, q.delay_C, q.drop_R, q.drop_C, 0.03)
        if r % 25 == 24:
            st = a.state()
            assert np.array_equal(st["t"], b.t) and np.array_equal(st["tau_v"], b.tau_v)
            assert np.array_equal(st["tau_rho"], b.tau_rho)
            for k, ref in (("x", b.x), ("z", b.z), ("g", b.g)):
                np.testing.assert_allclose(st[k], ref, rtol=1e-11, atol=1e-12)
    with pytest.raises(ValueError):
        a.round(q.active, q.delay_R + D, q.delay_C, q.drop_R, q.drop_C, 0.03)


def test_lemma3_and_closed_form_limit():
    n, p = 8, 5
    wr, wc = graphs.bidirectional_ring(n)
    R, C = graphs.from_dense(wr, fp32_weights=False), graphs.from_dense(wc, fp32_weights=False)
    rng = np.random.default_rng(3)
    h, c = rng.uniform(0.5, 2.0, (n, p)), rng.standard_normal((n, p))
    orc = COracle(n, p, R, C, 7, 4, h, c)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, np.full(n, 0.6), 4, 0.15, seed=1)
    for r in range(5000):
        q = sched.round(r)
        orc.round(q.active, q.delay_R, q.delay_C, q.drop_R, q.drop_C, 0.12)
        if r % 500 == 0:
            st = orc.state()
            res = st["z"].sum(0) - st["g"].sum(0)
            for e in range(orc.eC):
                rho, rt = orc.edge(e)
                res = res + rho - rt
            assert np.abs(res).max() < 1e-11
    st = orc.state()
    x_star = (h * c).sum(0) / h.sum(0)
    assert np.abs(st["x"] - x_star).max() < 1e-8 and np.abs(st["z"]).max() < 1e-8
