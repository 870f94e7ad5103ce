"""Pins of the fp64 oracle against what the paper and the mathematics fix.
None of these tests touches the GPU or the HIP library."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle.objectives import DiagQuadratic, LeastSquares
from oracle.rfast_oracle import RFastOracle
from rfast_workloads import configs, graphs
from rfast_workloads.schedule import ScheduleSpec

from dense_augmented import DenseAugmented

HERE = os.path.dirname(os.path.abspath(__file__))


def _random_problem(n, p, seed, noise=0.0):
    rng = np.random.default_rng(seed)
    h = rng.uniform(0.5, 2.0, (n, p))
    c = rng.standard_normal((n, p)) + np.arange(n)[:, None] / n
    return DiagQuadratic(h, c, noise, 99), h, c


def _run(orc, sched, rounds, gamma, every=None):
    for r in range(rounds):
        q = sched.round(r)
        orc.round(q.active, q.delay_R, q.delay_C, q.drop_R, q.drop_C, gamma, q.batch_idx)
        if every is not None:
            every(r, orc)


# ---------------------------------------------------------------- worked example
def _parse_golden():
    rows = []
    with open(os.path.join(HERE, "golden", "n3_ring_worked_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            cols = [c.strip() for c in line.split("|")]
            fr = lambda s: [float(Fraction(tok)) for tok in s.split()]
            zh = {int(a.split(":")[0]): float(Fraction(a.split(":")[1])) for a in cols[7].split()}
            rows.append(dict(x=fr(cols[1]), z=fr(cols[2]), g=fr(cols[3]), rho=fr(cols[4]),
                             rho_t=fr(cols[5]), t=[int(v) for v in cols[6].split()], zh=zh))
    return rows


def test_hand_stepped_n3_example_exact():
    """Algorithm 2 stepped by hand (golden file); every value is a dyadic
    rational, so the fp64 oracle must reproduce it exactly."""
    r, c = graphs.directed_ring(3)
    R, C = graphs.from_dense(r), graphs.from_dense(c)
    assert R.off_edges() == [(0, 2), (1, 0), (2, 1)]
    obj = DiagQuadratic(np.array([[1.0], [2.0], [1.0]]), np.array([[1.0], [2.0], [4.0]]))
    orc = RFastOracle(3, 1, R, C, D=2, burst=2, objective=obj)
    assert orc.z[:, 0].tolist() == [-1.0, -4.0, -4.0]
    gold = _parse_golden()
    # edge ids in CSR order: e0 = (0<-2), e1 = (1<-0), e2 = (2<-1); golden order is (1,0),(2,1),(0,2)
    perm = [1, 2, 0]
    sched = [
        dict(active=[1, 1, 0], dR=[0, 0, 0], dC=[0, 0, 0], xR=[0, 0, 0], xC=[0, 0, 1]),
        dict(active=[0, 1, 1], dR=[0, 1, 0], dC=[0, 1, 0], xR=[0, 0, 0], xC=[0, 0, 0]),
        dict(active=[1, 1, 1], dR=[0, 0, 0], dC=[0, 0, 0], xR=[0, 0, 0], xC=[0, 0, 0]),
    ]
    stamps = [
        {0: ({0: 0}, {0: 0}), 1: ({1: 0}, {1: 0})},
        {1: ({1: 0}, {1: 0}), 2: ({2: 1}, {2: 0})},
        {0: ({0: 1}, {0: 1}), 1: ({1: 1}, {1: 1}), 2: ({2: 2}, {2: 2})},
    ]
    for k, (s, gd) in enumerate(zip(sched, gold)):
        for i, (sv, sr) in stamps[k].items():
            assert orc.resolve(i, s["dR"], s["dC"]) == (sv, sr), (k, i)
        orc.round(s["active"], s["dR"], s["dC"], s["xR"], s["xC"], 0.25)
        assert orc.x[:, 0].tolist() == gd["x"], k
        assert orc.z[:, 0].tolist() == gd["z"], k
        assert orc.g[:, 0].tolist() == gd["g"], k
        assert orc.t.tolist() == gd["t"], k
        latest = [orc.rho[e][int(orc.t[orc.edges_C[e][1]])][0] for e in perm]
        assert latest == gd["rho"], k
        assert [orc.rho_tilde[e][0] for e in perm] == gd["rho_t"], k
        for i, v in gd["zh"].items():
            assert orc.last_z_half[i, 0] == v, (k, i)
        assert orc.conservation_residual()[0] == 0.0


# ------------------------------------------------------- invariants (Lemma 3 etc.)
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_tracking_conservation_and_running_sum(seed):
    """Lemma 3: sum z + in-flight mass = sum of stored gradient samples, every
    round, for any schedule with delays, losses and gradient noise.  Also the
    closed form rho_ij = a_ij * (sum of all z_half node j ever produced)."""
    n, p = 7, 5
    rng = np.random.default_rng(seed)
    wr, wc = graphs.random_digraph(n, rng)
    R, C = graphs.from_dense(wr, fp32_weights=False), graphs.from_dense(wc, fp32_weights=False)
    obj, _, _ = _random_problem(n, p, seed, noise=0.3)
    orc = RFastOracle(n, p, R, C, D=6, burst=3, objective=obj, x0=rng.standard_normal((n, p)))
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, np.full(n, 0.6), 4, 0.3, seed=seed)
    zsum = np.zeros((n, p))
    scale = [1.0]

    def check(r, o):
        act = sched.round(r).active
        for i in range(n):
            if act[i]:
                zsum[i] += o.last_z_half[i]
        scale[0] = max(scale[0], np.abs(zsum).max())
        assert np.abs(o.conservation_residual()).max() <= 1e-12 * scale[0] * n
        for e, (i, j) in enumerate(o.edges_C):
            a_ij = C.dense()[i, j]
            np.testing.assert_allclose(o.rho[e][int(o.t[j])], a_ij * zsum[j], rtol=0, atol=1e-12 * scale[0])

    _run(orc, sched, 120, 0.05, check)


def test_resolver_properties_and_mailbox_bruteforce():
    """Stamps are monotone, never newer than what the sender had published
    before round r-d, never staler than D versions, never a lost version; and
    they equal a brute-force simulation with explicit packets and mailboxes."""
    n, p, d_max, burst = 6, 1, 3, 3
    D = d_max + burst - 1
    rng = np.random.default_rng(5)
    wr, wc = graphs.random_digraph(n, rng, extra=0.4)
    R, C = graphs.from_dense(wr), graphs.from_dense(wc)
    obj, _, _ = _random_problem(n, p, 1)
    orc = RFastOracle(n, p, R, C, D=D, burst=burst, objective=obj)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, np.full(n, 0.5), d_max, 0.45, seed=3)
    edges = {"R": R.off_edges(), "C": C.off_edges()}
    # brute force: packets[kind][e] = list of (sent_round, stamp) actually delivered
    packets = {k: [[] for _ in edges[k]] for k in "RC"}
    lost_run = {k: [0] * len(edges[k]) for k in "RC"}
    held = {k: [0] * len(edges[k]) for k in "RC"}
    t = [0] * n
    n_forced = 0
    for r in range(300):
        q = sched.round(r)
        delays = {"R": q.delay_R, "C": q.delay_C}
        drops = {"R": q.drop_R, "C": q.drop_C}
        expect = {}
        for kind in "RC":
            for e, (i, j) in enumerate(edges[kind]):
                if not q.active[i]:
                    continue
                visible = [st for (sr, st) in packets[kind][e] if sr < r - delays[kind][e]]
                held[kind][e] = max([held[kind][e]] + visible)
                expect[(kind, e)] = held[kind][e]
        prev = {"R": orc.tau_v.copy(), "C": orc.tau_rho.copy()}
        t_before = orc.t.copy()
        orc.round(q.active, q.delay_R, q.delay_C, q.drop_R, q.drop_C, 0.01)
        now = {"R": orc.tau_v, "C": orc.tau_rho}
        for (kind, e), st in expect.items():
            i, j = edges[kind][e]
            assert now[kind][e] == st
            assert now[kind][e] >= prev[kind][e]
            assert t_before[j] - D <= now[kind][e] <= t_before[j]
        # senders publish after all reads of the round
        for kind in "RC":
            for e, (i, j) in enumerate(edges[kind]):
                if q.active[j]:
                    lost = bool(drops[kind][e]) and lost_run[kind][e] < burst - 1
                    n_forced += bool(drops[kind][e]) and not lost
                    if lost:
                        lost_run[kind][e] += 1
                    else:
                        lost_run[kind][e] = 0
                        packets[kind][e].append((r, t[j] + 1))
        for j in range(n):
            t[j] += int(q.active[j])
        assert t == orc.t.tolist()
    assert n_forced > 10  # the forced-delivery rule was exercised


def test_serialisation_equivalence():
    """A batched round equals its active nodes' single activations applied one
    after the other in any order (each reads only versions published before
    the round and writes only its own state): bit-exact."""
    n, p = 8, 4
    rng = np.random.default_rng(11)
    wr, wc = graphs.random_digraph(n, rng)
    R, C = graphs.from_dense(wr), graphs.from_dense(wc)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, np.full(n, 0.7), 3, 0.2, seed=8)
    orcs = []
    for variant in range(3):
        obj, _, _ = _random_problem(n, p, 4, noise=0.1)
        orcs.append(RFastOracle(n, p, R, C, D=5, burst=3, objective=obj))
    for r in range(60):
        q = sched.round(r)
        act = [i for i in range(n) if q.active[i]]
        orders = [None, act[::-1], list(np.random.default_rng(r).permutation(act))]
        for o, order in zip(orcs, orders):
            o.round(q.active, q.delay_R, q.delay_C, q.drop_R, q.drop_C, 0.03, None, order=order)
        for o in orcs[1:]:
            assert np.array_equal(o.x, orcs[0].x) and np.array_equal(o.z, orcs[0].z)
            assert np.array_equal(o.tau_rho, orcs[0].tau_rho)
            for e in range(len(o.edges_C)):
                assert np.array_equal(o.rho_tilde[e], orcs[0].rho_tilde[e])


# ---------------------------------------------------- synchronous special case
def test_synchronous_reduction_matches_dense_recursion():
    """Remark 1: with every node active, zero delay and no loss the method is
    the synchronous push-pull recursion with a one-step communication lag:
      v^{r+1} = x^r - gamma z^r,  x^{r+1} = diag(W) v^{r+1} + offdiag(W) v^r,
      y^r = z^r + offdiag(A) y^{r-1} + g^{r+1} - g^r,  z^{r+1} = diag(A) y^r,
    written here with dense matrices only."""
    n, p, gamma = 6, 3, 0.07
    rng = np.random.default_rng(2)
    wr, wc = graphs.random_digraph(n, rng)
    R, C = graphs.from_dense(wr, fp32_weights=False), graphs.from_dense(wc, fp32_weights=False)
    obj, h, c = _random_problem(n, p, 3)
    x0 = rng.standard_normal((n, p))
    orc = RFastOracle(n, p, R, C, D=1, burst=1, objective=obj, x0=x0)
    Wd, Wo = np.diag(np.diag(wr)), wr - np.diag(np.diag(wr))
    Ad, Ao = np.diag(np.diag(wc)), wc - np.diag(np.diag(wc))
    x, g = x0.copy(), h * (x0 - c)
    z, v_prev, y_prev = g.copy(), np.zeros((n, p)), np.zeros((n, p))
    ones, zeros = np.ones(n, np.uint8), np.zeros(R.nnz_off, np.int32)
    zc = np.zeros(C.nnz_off, np.int32)
    for r in range(40):
        orc.round(ones, zeros, zc, zeros.astype(np.uint8), zc.astype(np.uint8), gamma)
        v = x - gamma * z
        x = Wd @ v + Wo @ v_prev
        g_new = h * (x - c)
        y = z + Ao @ y_prev + g_new - g
        z = Ad @ y
        g, v_prev, y_prev = g_new, v, y
        np.testing.assert_allclose(orc.x, x, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(orc.z, z, rtol=1e-12, atol=1e-13)


# ------------------------------------------------- augmented-system formulation
@pytest.mark.parametrize("seed", [0, 1])
def test_dense_augmented_system_cross_formulation(seed):
    """Single-node activations with delays (Algorithm 2) against the paper's
    augmented matrices: W-hat^k must be row-stochastic, S^k and P^k column-
    stochastic, and x, z and the in-flight edge masses must agree."""
    n, p, D, gamma = 4, 2, 3, 0.05
    rng = np.random.default_rng(100 + seed)
    wr, wc = graphs.random_digraph(n, rng, extra=0.35)
    R, C = graphs.from_dense(wr, fp32_weights=False), graphs.from_dense(wc, fp32_weights=False)
    obj, h, c = _random_problem(n, p, seed)
    x0 = rng.standard_normal((n, p))
    orc = RFastOracle(n, p, R, C, D=10 ** 6, burst=1, objective=obj, x0=x0, prune=False)
    dense = DenseAugmented(wr, wc, D, x0, h * (x0 - c))
    assert dense.edges == C.off_edges()
    grad = lambda i, x: h[i] * (x - c[i])
    t_at = [np.zeros(n, dtype=int)]          # t_at[k][j]: activations of j before global iteration k
    last_read = {ed: 0 for ed in C.off_edges()}
    eR = {ed: k for k, ed in enumerate(R.off_edges())}
    eC = {ed: k for k, ed in enumerate(C.off_edges())}
    for k in range(80):
        i = int(rng.integers(n))
        d_v = {j: int(rng.integers(0, D + 1)) for (ii, j) in R.off_edges() if ii == i}
        d_rho = {}
        for (ii, j) in C.off_edges():
            if ii == i:
                lo = max(last_read[(i, j)], k - D)
                read_time = int(rng.integers(lo, k + 1))
                d_rho[j] = k - read_time
                last_read[(i, j)] = read_time
        Wh, Sm, Pm = dense.step(i, d_v, d_rho, gamma, grad)
        np.testing.assert_allclose(Wh.sum(axis=1), 1.0, atol=1e-14)
        np.testing.assert_allclose(Sm.sum(axis=0), 1.0, atol=1e-14)
        np.testing.assert_allclose(Pm.sum(axis=0), 1.0, atol=1e-14)
        sv = {eR[(i, j)]: int(t_at[max(k - d, 0)][j]) for j, d in d_v.items()}
        sr = {eC[(i, j)]: int(t_at[max(k - d, 0)][j]) for j, d in d_rho.items()}
        orc.activate(i, sv, sr, gamma)
        nxt = t_at[-1].copy()
        nxt[i] += 1
        t_at.append(nxt)
        np.testing.assert_allclose(orc.x, dense.h[:n], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(orc.z, dense.zhat[:n], rtol=1e-12, atol=1e-13)
        vk = np.stack([orc.v[j][int(orc.t[j])] for j in range(n)])
        np.testing.assert_allclose(vk, dense.h[n:2 * n], rtol=1e-12, atol=1e-13)
        for e, (ii, j) in enumerate(C.off_edges()):
            inflight = sum(dense.zhat[dense.vnode(e, d)] for d in range(D + 1))
            np.testing.assert_allclose(orc.rho[e][int(orc.t[j])] - orc.rho_tilde[e], inflight,
                                       rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(dense.zhat.sum(axis=0), orc.g.sum(axis=0), rtol=1e-12, atol=1e-12)


# ----------------------------------------------------------------- fixed points
def test_fixed_point_least_squares_closed_form():
    """Theorem 1 with sigma = 0: geometric convergence to the minimiser of
    F = sum_i f_i, x* = (sum A_i^T A_i)^-1 sum A_i^T b_i, over a directed ring
    with delays and losses, although every node's own optimum differs."""
    w = configs.config0(p=4, m=12, rounds=0)           # graph and schedule law of config 0
    rng = np.random.default_rng(0)
    n, p, m = w.n, 4, 12
    A = rng.standard_normal((n, m, p))                 # each node has its own teacher
    b = np.einsum("imp,ip->im", A, rng.standard_normal((n, p))) + 0.1 * rng.standard_normal((n, m))
    H = sum(A[i].T @ A[i] for i in range(n))
    x_star = np.linalg.solve(H, sum(A[i].T @ b[i] for i in range(n)))
    local = np.stack([np.linalg.lstsq(A[i], b[i], rcond=None)[0] for i in range(n)])
    assert np.abs(local - x_star).max() > 0.3           # heterogeneous shards
    orc = RFastOracle(n, p, w.R, w.C, w.D, w.burst, LeastSquares(A, b))
    errs = []
    _run(orc, w.sched, 9000, 0.04, lambda r, o: errs.append(np.abs(o.x - x_star).max()) if r % 1000 == 999 else None)
    assert errs[-1] < 1e-8, errs
    assert np.abs(orc.z).max() < 1e-7
    # geometric: equal-length windows shrink by a roughly constant factor
    ratios = [errs[k + 1] / errs[k] for k in range(1, 7)]
    assert all(0.01 < rt < 0.3 for rt in ratios), errs


def test_named_topologies_satisfy_assumption_1_and_2():
    """Row- / column-stochastic with positive diagonal, weights from the degrees, and the common
    roots the construction promises (reachability by brute force on the dense matrices)."""
    def reach(adj, src):          # nodes that hear src, directly or not (adj[i, j]: i hears j)
        seen, todo = {src}, [src]
        while todo:
            j = todo.pop()
            for i in np.nonzero(adj[:, j])[0]:
                if int(i) not in seen:
                    seen.add(int(i)); todo.append(int(i))
        return seen
    cases = [(graphs.binary_tree(7), {0}), (graphs.binary_tree(12), {0}), (graphs.mesh(9), set(range(9))),
             (graphs.mesh(7), set(range(7))), (graphs.multi_root_split(11, 3), {0, 1, 2}),
             (graphs.line_tree(5), {0}), (graphs.directed_ring(4), set(range(4)))]
    for (wr, wc), roots in cases:
        n = wr.shape[0]
        assert np.allclose(wr.sum(axis=1), 1) and np.allclose(wc.sum(axis=0), 1)
        assert (np.diag(wr) > 0).all() and (np.diag(wc) > 0).all() and (wr >= 0).all() and (wc >= 0).all()
        for m in (wr, wc):   # uniform over the non-zeros of a row of R / a column of C
            nz = m != 0
            assert np.allclose(m[nz], (nz / nz.sum(axis=1, keepdims=True))[nz] if m is wr
                               else (nz / nz.sum(axis=0, keepdims=True))[nz])
        # root of G(R): everybody hears it through R; root of G(C^T): it hears everybody through C
        got = {j for j in range(n) if len(reach(wr != 0, j)) == n and len(reach((wc != 0).T, j)) == n}
        assert got == roots, (got, roots)


@pytest.mark.parametrize("topology", ["tree_star", "biring", "exp", "binary_tree", "mesh", "multi_root"])
def test_fixed_point_diag_quadratic_closed_form(topology):
    """x*_k = sum_i h_ik c_ik / sum_i h_ik, reached over spanning-tree graphs
    that are not strongly connected (Assumption 2) as well."""
    n, p = 8, 6
    wr, wc = {"tree_star": graphs.tree_pull_star_push, "biring": graphs.bidirectional_ring,
              "exp": graphs.exponential, "binary_tree": graphs.binary_tree, "mesh": graphs.mesh,
              "multi_root": lambda m: graphs.multi_root_split(m, 3)}[topology](n)
    # exact weights: with fp32-rounded thirds the columns of C sum to 1 + 3e-8 and
    # the tracker leaks that share of every z_half, which moves the limit by ~1e-6
    R, C = graphs.from_dense(wr, fp32_weights=False), graphs.from_dense(wc, fp32_weights=False)
    obj, h, c = _random_problem(n, p, 21)
    x_star = (h * c).sum(axis=0) / h.sum(axis=0)
    gamma = {"tree_star": 0.01, "biring": 0.12, "exp": 0.15, "binary_tree": 0.01, "mesh": 0.12, "multi_root": 0.03}[topology]
    orc = RFastOracle(n, p, R, C, D=7, burst=4, objective=obj)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, np.full(n, 0.6), 4, 0.15, seed=1)
    _run(orc, sched, 6000, gamma)
    assert np.abs(orc.x - x_star).max() < 1e-8
    assert np.abs(orc.z).max() < 1e-8


def test_sample_stamp_convention():
    """The sample of the initial gradient has stamp 0, the one drawn at a node's
    t-th activation has stamp t (the node's local iteration counter): with h = 0
    the stored gradient is the noise alone."""
    from oracle.objectives import gaussian_noise
    n, p = 4, 8
    wr, wc = graphs.directed_ring(n)
    R, C = graphs.from_dense(wr), graphs.from_dense(wc)
    obj = DiagQuadratic(np.zeros((n, p)), np.zeros((n, p)), 0.5, 31)
    orc = RFastOracle(n, p, R, C, D=4, burst=2, objective=obj)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, np.full(n, 0.5), 3, 0.2, seed=2)
    for i in range(n):
        np.testing.assert_array_equal(orc.g[i], 0.5 * gaussian_noise(31, i, 0, p))
    _run(orc, sched, 25, 0.1)
    assert len(set(orc.t.tolist())) > 1
    for i in range(n):
        np.testing.assert_array_equal(orc.g[i], 0.5 * gaussian_noise(31, i, int(orc.t[i]), p))


def test_noise_floor_scales_with_sigma():
    """Theorem 1: with gradient noise the iterates settle in a neighbourhood of
    x* whose squared radius is proportional to sigma^2."""
    n, p = 8, 64
    wr, wc = graphs.bidirectional_ring(n)
    R, C = graphs.from_dense(wr), graphs.from_dense(wc)
    res = []
    for std in (0.05, 0.2):
        obj, h, c = _random_problem(n, p, 5, noise=std)
        x_star = (h * c).sum(axis=0) / h.sum(axis=0)
        orc = RFastOracle(n, p, R, C, D=7, burst=4, objective=obj)
        sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, np.full(n, 1.0), 4, 0.02, seed=1)
        acc = []
        _run(orc, sched, 3000, 0.15, lambda r, o: acc.append(((o.x - x_star) ** 2).mean()) if r >= 2000 else None)
        res.append(np.mean(acc))
    assert 8.0 < res[1] / res[0] < 32.0, res   # (0.2/0.05)^2 = 16
