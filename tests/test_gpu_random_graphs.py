"""GPU parity on random instances: random digraphs with non-dyadic weights and
uneven degrees (in-degrees above the kernel's load batch of 8), random
schedules, extreme ring depths and burst settings."""
import numpy as np
import pytest

from rfast_workloads import configs, graphs, problems
from rfast_workloads.schedule import ScheduleSpec

import harness

pytestmark = pytest.mark.gpu


def _workload(n, p, wr, wc, d_max, burst, p_active, p_drop, seed, gamma=0.03, noise=0.05):
    R, C = graphs.from_dense(wr), graphs.from_dense(wc)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, np.full(n, p_active), d_max, p_drop, seed=seed)
    return configs.Workload(f"random_n{n}_p{p}_s{seed}", n, p, R, C, d_max + burst - 1, burst, gamma, 0,
                            "diag_quadratic", problems.diag_quadratic(n, p, seed), sched, noise, 777 + seed, 1e-4)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_digraph(seed):
    rng = np.random.default_rng(seed)
    n = [5, 13, 24][seed]
    wr, wc = graphs.random_digraph(n, rng, extra=[0.3, 0.5, 0.6][seed])
    w = _workload(n, [1028, 260, 516][seed], wr, wc, d_max=[2, 5, 3][seed], burst=[1, 3, 5][seed],
                  p_active=[0.9, 0.5, 0.3][seed], p_drop=[0.5, 0.3, 0.4][seed], seed=seed)
    assert (wr != 0).sum(axis=1).max() - 1 > 8 or seed == 0
    worst, orc, gpu = harness.run_parity(w, 240, every=60)
    print(f"\n[{w.name}] worst {worst}")


@pytest.mark.parametrize("name", ["binary_tree", "line", "mesh", "multi_root", "directed_ring", "exponential"])
def test_named_topologies(name):
    """The topologies of the experiments on general graphs (trees and lines as a pull tree and
    its inverse, which are not strongly connected) and the parameter-server-like split."""
    build, n = {"binary_tree": (graphs.binary_tree, 15), "line": (graphs.line_tree, 7), "mesh": (graphs.mesh, 11),
                "multi_root": (lambda m: graphs.multi_root_split(m, 3), 11), "directed_ring": (graphs.directed_ring, 7),
                "exponential": (graphs.exponential, 7)}[name]
    wr, wc = build(n)
    w = _workload(n, 1028, wr, wc, d_max=3, burst=2, p_active=0.6, p_drop=0.2, seed=n, gamma=0.01)
    worst, orc, gpu = harness.run_parity(w, 300, every=75)
    print(f"\n[{name} n={n}] worst {worst}")


def test_deepest_ring_and_dense_graph():
    """D + 2 = 64 slots (the bitmask limit), complete graph: 15 in- and out-edges per node."""
    n = 16
    rng = np.random.default_rng(9)
    wr, wc = graphs.random_digraph(n, rng, extra=1.1)
    w = _workload(n, 132, wr, wc, d_max=40, burst=23, p_active=0.7, p_drop=0.8, seed=9)
    assert w.D == 62
    worst, orc, gpu = harness.run_parity(w, 400, every=100)
    print(f"\n[{w.name}] worst {worst}")


def test_no_delay_no_loss_is_synchronous_special_case():
    """Remark 1: every node active, zero delay, nothing lost; D = 0 gives a two-slot ring."""
    n = 6
    wr, wc = graphs.exponential(n)
    w = _workload(n, 2048, wr, wc, d_max=0, burst=1, p_active=1.0, p_drop=0.0, seed=4, gamma=0.08, noise=0.0)
    assert w.D == 0
    worst, orc, gpu = harness.run_parity(w, 150, every=50)
    d = gpu.diagnostics()
    assert d["consensus_sq"] < 1e-3 * w.p     # the nodes agree
    print(f"\n[{w.name}] worst {worst}")


def test_many_nodes_tiny_vectors():
    """n above the resolver's workgroup size (active-list compaction and edge loops in
    several chunks), p = 3 (scalar path, one partial tile)."""
    n = 1500
    rng = np.random.default_rng(3)
    adj = np.eye(n, dtype=bool)
    for j in range(n):
        adj[(j + 1) % n, j] = True
        for t in rng.integers(0, n, 2):
            adj[t, j] = True
    wr = adj / adj.sum(axis=1, keepdims=True)
    wc = adj / adj.sum(axis=0, keepdims=True)
    w = _workload(n, 3, wr, wc, d_max=3, burst=2, p_active=0.4, p_drop=0.2, seed=5, gamma=0.05, noise=0.1)
    assert w.R.nnz_off > 2048
    worst, orc, gpu = harness.run_parity(w, 60, every=20)
    print(f"\n[{w.name}] worst {worst}")


def test_single_coordinate_and_full_batch_logistic():
    w = configs.config1(p=1, samples=64, batch=64, rounds=0)
    worst, orc, gpu = harness.run_parity(w, 120, every=40)
    print(f"\n[{w.name} p=1 full batch] worst {worst}")


def test_buffers_that_leave_the_senders_ring():
    """The S4 buffer rho~ is kept implicitly (the sender's ring still holds that version) or in
    its own array (the version has left the ring).  Shallow ring, always-active senders and
    rarely active receivers: every way of handing a buffer over occurs, and every buffer read
    back equals the oracle's (run_parity compares rho~ of every edge at every checkpoint)."""
    n = 10
    rng = np.random.default_rng(21)
    wr, wc = graphs.random_digraph(n, rng, extra=0.6)
    R, C = graphs.from_dense(wr), graphs.from_dense(wc)
    p_act = np.where(np.arange(n) % 3 == 0, 0.15, 1.0)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, p_act, 1, 0.3, seed=5)
    w = configs.Workload("shallow_ring_lagging_receivers", n, 260, R, C, 1 + 2 - 1, 2, 0.01, 0, "diag_quadratic",
                         problems.diag_quadratic(n, 260, 5), sched, 0.05, 31, 1e-4)
    assert w.D == 2
    worst, orc, gpu = harness.run_parity(w, 300, every=20)
    # at the end: buffers inside the ring window, on its edge, and outside it all exist
    lag = np.array([int(orc.t[j]) - int(orc.tau_rho[e]) for e, (i, j) in enumerate(orc.edges_C)])
    assert (lag < w.D).any() and (lag == w.D).any() and (lag > w.D).any(), lag
    d = gpu.diagnostics()
    assert d["conservation_sq"] <= 1e-8 * max(d["gsum_sq"], 1.0)
    print(f"\n[{w.name}] worst {worst}, lags {np.bincount(np.minimum(lag, 8))}")


@pytest.mark.parametrize("seed", list(range(100, 112)))
def test_random_configuration_sweep(seed):
    """Seeded random draws of everything at once: size, ring depth, burst bound, activity (uniform
    or with near-idle nodes), loss rate, delays, vector length (float4 and scalar paths), step size.
    Every checkpoint compares stamps, slots, x, z, g, the v and rho rings and the S4 buffers."""
    rng = np.random.default_rng(seed)
    n = int(rng.integers(2, 20))
    p = int(rng.choice([1, 3, 4, 64, 130, 257, 516]))
    d_max = int(rng.integers(0, 7))
    burst = int(rng.integers(1, 6))
    wr, wc = graphs.random_digraph(n, rng, extra=float(rng.uniform(0.0, 1.0)))
    R, C = graphs.from_dense(wr), graphs.from_dense(wc)
    p_act = rng.uniform(0.05, 1.0, n) if seed % 2 else np.full(n, float(rng.uniform(0.2, 1.0)))
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, p_act, d_max, float(rng.uniform(0.0, 0.9)), seed=seed)
    w = configs.Workload(f"sweep_{seed}", n, p, R, C, d_max + burst - 1, burst, float(rng.uniform(0.005, 0.04)), 0,
                         "diag_quadratic", problems.diag_quadratic(n, p, seed), sched, float(rng.choice([0.0, 0.1])),
                         1000 + seed, 1e-4)
    x0 = rng.standard_normal((n, p)).astype(np.float32) if seed % 3 == 0 else None
    worst, orc, gpu = harness.run_parity(w, 160, every=20, x0=x0)
    d = gpu.diagnostics()
    assert d["conservation_sq"] <= 1e-7 * max(d["gsum_sq"], d["z_sq"], 1.0)


@pytest.mark.parametrize("seed", list(range(200, 208)))
def test_random_configuration_sweep_sampled_gradients(seed):
    """The same kind of sweep on the split path (mix, gradient kernels, track): least squares with
    full local gradients and logistic regression with minibatches, random sizes incl. odd p."""
    rng = np.random.default_rng(seed)
    n = int(rng.integers(2, 14))
    p = int(rng.choice([5, 64, 132, 259, 1028]))
    d_max = int(rng.integers(0, 6))
    burst = int(rng.integers(1, 5))
    wr, wc = graphs.random_digraph(n, rng, extra=float(rng.uniform(0.0, 0.8)))
    p_act = rng.uniform(0.1, 1.0, n)
    if seed % 2:
        m = int(rng.integers(3, 40))
        w = configs._mk(f"sweep_ls_{seed}", n, p, wr, wc, d_max, 0.4 / p, 0, "least_squares",
                        problems.least_squares(n, p, m, seed), p_act, float(rng.uniform(0, 0.6)), seed, samples=m, burst=burst)
    else:
        samples = int(rng.integers(8, 80))
        batch = int(rng.integers(1, samples + 1))
        w = configs._mk(f"sweep_logistic_{seed}", n, p, wr, wc, d_max, 0.05, 0, "logistic",
                        problems.logistic(n, p, samples, seed), p_act, float(rng.uniform(0, 0.6)), seed, batch=batch,
                        samples=samples, burst=burst)
    worst, orc, gpu = harness.run_parity(w, 120, every=30)
