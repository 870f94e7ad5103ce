"""Several rounds per launch with the per-coordinate state resident in LDS must give the same bits
as one kernel pass per round: same plans, same arithmetic, only the memory the values travel
through differs.  Uploaded and generated schedules, launches cut short by the rebase interval
and by the step-size schedule, graphs whose rings spill S4 buffers, ragged last tile."""
import numpy as np
import pytest
import torch

from paper_2307_11617_amd import rfast_block_info, rfast_use_blocks, rfast_set_rebase_interval
from rfast_workloads import configs, graphs, problems
from rfast_workloads.schedule import ScheduleSpec

import harness

pytestmark = pytest.mark.gpu
FIELDS = ("X", "Z", "G", "V_RING", "SIGMA_RING", "RHO_TILDE", "T_NODE", "TAU_R", "TAU_C", "SLOT_R", "SLOT_C", "ROUND")
INTEGER_REST = ("DELIV_R", "DELIV_C", "T_HIST")   # what else a resolver leaves behind (the kernel of small graphs has its own)


def _pair(w):
    a, b = harness.make_gpu(w), harness.make_gpu(w)
    rfast_use_blocks(b.ctx, False)
    return a, b


def _same(a, b, where, more=()):
    for f in FIELDS + tuple(more):
        assert np.array_equal(a.read(f), b.read(f)), (where, f)


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4, 5, 6])
def test_uploaded_schedules(seed):
    """Seeds 1-3: random graphs with at most four edges of a kind per node; seed 4 has six (the widest kernel of the
    tile-per-wavefront path); seed 5 has eight, and must run one pass per round; seed 6: the exponential graph on
    32 nodes (five edges of a kind per node, two lanes per node)."""
    rng = np.random.default_rng(seed)
    n = [16, 5, 33, 9, 9, 9, 32][seed]
    p = [1028, 64, 260, 4100, 512, 512, 1036][seed]
    d_max, burst = [4, 0, 2, 1, 1, 1, 3][seed], [4, 1, 2, 3, 2, 2, 3][seed]
    if seed == 0:
        wr, wc = graphs.bidirectional_ring(n)
    elif seed == 6:
        wr, wc = graphs.exponential(n)
    else:
        wr, wc = graphs.random_digraph(n, rng, extra=[0, 0.4, 0.02, 0.2, 0.4, 0.8][seed])
    R, C = graphs.from_dense(wr), graphs.from_dense(wc)
    p_act = np.where(np.arange(n) % 4 == 1, 0.1, 0.9)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, p_act, d_max, 0.3, seed=seed)
    w = configs.Workload(f"blocks_{seed}", n, p, R, C, d_max + burst - 1, burst, 0.02, 0, "diag_quadratic",
                         problems.diag_quadratic(n, p, seed), sched, 0.1, 50 + seed, 1e-4)
    a, b = _pair(w)
    off = lambda m: (m != 0) & ~np.eye(n, dtype=bool)
    degree = max(off(wr).sum(1).max(), off(wc).sum(1).max(), off(wc).sum(0).max())   # in R, in C, out C
    assert degree == [2, 3, 4, 4, 6, 8, 5][seed]
    assert (rfast_block_info(a.ctx) != 0) == (degree <= (6 if n <= 32 else 4)), degree
    x0 = rng.standard_normal((n, p)).astype(np.float32)
    for g in (a, b):
        rfast_set_rebase_interval(g.ctx, 23)       # launches end on multiples of 23
        g.set_gamma_schedule(10, 0.7)
        g.init(x0, None)
    st, dev = harness.upload_chunk(a, w, 0, 75)
    cut = lambda lo, hi: [dev[k][lo:hi] for k in ("active", "delay_R", "delay_C", "drop_R", "drop_C")]
    for lo, hi in ((0, 37), (37, 38), (38, 75)):   # a long call, a single round, another long call
        for g in (a, b):
            g.run(hi - lo, *cut(lo, hi), w.gamma)
            g.check()
        _same(a, b, (seed, hi))
    # and the result is the oracle's
    orc = harness.make_oracle(w, None, x0)
    from oracle.rfast_oracle import step_gamma
    for r in range(75):
        orc.round(st["active"][r], st["delay_R"][r], st["delay_C"][r], st["drop_R"][r], st["drop_C"][r],
                  step_gamma(w.gamma, 0.7, 10, r))
    assert harness.rel_l2(a.read("X"), orc.x) <= 1e-4
    assert harness.rel_l2(a.read("Z"), orc.z, 1e-3 * float(np.linalg.norm(orc.g))) <= 1e-4
    assert np.array_equal(a.read("T_NODE"), orc.t)


# n, d_max, burst, p, lanes per node the library must choose: up to 32 nodes one tile per wavefront
# (64 // n lanes per node); beyond, one tile per workgroup (the widest that fits LDS and 1024 lanes and
# leaves 512 tiles, from 64, 48, 32, 28, 24, 16); every p ends in a ragged tile
TILES = [(16, 4, 4, 65_540, 4), (16, 5, 4, 49_156, 4), (5, 0, 1, 131_076, 12), (9, 3, 4, 98_308, 7),
         (14, 7, 4, 57_348, 4), (24, 1, 2, 65_540, 2), (32, 2, 2, 8_196, 2), (16, 4, 4, 4_100, 4),
         (1, 0, 1, 4_100, 64), (2, 1, 1, 4_100, 32), (3, 1, 2, 4_100, 21),
         (36, 0, 1, 57_348, 28), (40, 0, 1, 49_156, 24), (48, 1, 1, 8_196, 16)]


@pytest.mark.parametrize("n,d_max,burst,p,lanes", TILES)
def test_tile_widths(n, d_max, burst, p, lanes):
    wr, wc = graphs.bidirectional_ring(n)
    R, C = graphs.from_dense(wr), graphs.from_dense(wc)
    p_act = np.where(np.arange(n) % 3 == 1, 0.3, 0.9)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, p_act, d_max, 0.3, seed=n)
    w = configs.Workload(f"tiles_{lanes}", n, p, R, C, d_max + burst - 1, burst, 0.02, 0, "diag_quadratic",
                         problems.diag_quadratic(n, p, n), sched, 0.1, 90 + n, 1e-4)
    a, b = _pair(w)
    assert rfast_block_info(a.ctx, with_kind=True) == (lanes, n <= 32) and rfast_block_info(b.ctx) == 0
    for g in (a, b):
        g.init(None, None)
    st, dev = harness.upload_chunk(a, w, 0, 40)
    args = [dev[k] for k in ("active", "delay_R", "delay_C", "drop_R", "drop_C")]
    for g in (a, b):
        g.run(40, *args, w.gamma)
        g.check()
    _same(a, b, lanes)


@pytest.mark.parametrize("n,d_max,burst,wave", [(8, 12, 4, True), (4, 29, 4, False)])
def test_deep_rings(n, d_max, burst, wave):
    """Rings of 17 slots, which the multi-round kernel moves in two batches, and of 34 slots, one more than the
    records of the resolver have bits for: those rounds go to the other kernels.  Same bits either way."""
    wr, wc = graphs.bidirectional_ring(n)
    R, C = graphs.from_dense(wr), graphs.from_dense(wc)
    p = 16_388
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, np.full(n, 0.7), d_max, 0.3, seed=n)
    w = configs.Workload(f"deep_{n}", n, p, R, C, d_max + burst - 1, burst, 0.02, 0, "diag_quadratic",
                         problems.diag_quadratic(n, p, n), sched, 0.1, 70 + n, 1e-4)
    a, b = _pair(w)
    assert rfast_block_info(a.ctx, with_kind=True)[1] == wave and rfast_block_info(b.ctx) == 0
    for g in (a, b):
        g.init(None, None)
    st, dev = harness.upload_chunk(a, w, 0, 60)
    cut = lambda lo, hi: [dev[k][lo:hi] for k in ("active", "delay_R", "delay_C", "drop_R", "drop_C")]
    for g in (a, b):
        g.run(45, *cut(0, 45), w.gamma)
        g.run(15, *cut(45, 60), w.gamma)
        g.check()
    _same(a, b, n)


def test_large_state_short_and_long_calls():
    """Above 8 MB of x a launch needs 8 rounds to pay: shorter calls run one pass per round, longer
    ones take the multi-round kernel (four refills of its plan records at 70 rounds), same bits."""
    w = configs.config2(p=131_076, rounds=0)
    a, b = _pair(w)
    for g in (a, b):
        g.init(None, None)
    st, dev = harness.upload_chunk(a, w, 0, 100)
    cut = lambda lo, hi: [dev[k][lo:hi] for k in ("active", "delay_R", "delay_C", "drop_R", "drop_C")]
    for lo, hi in ((0, 7), (7, 77), (77, 100)):
        for g in (a, b):
            g.run(hi - lo, *cut(lo, hi), w.gamma)
            g.check()
        _same(a, b, hi)


@pytest.mark.parametrize("n,variant", [(16, False), (16, True), (5, False), (24, True)])
def test_synchronous_steps_per_launch(n, variant):
    """rfast_sync_run through the multi-step kernel against one step per launch: same bits, with the
    optimizer variant and a step-size schedule that cuts the launches, a single step in between."""
    p = 4100
    wr, wc = graphs.bidirectional_ring(n) if n != 5 else graphs.exponential(n)
    R, C = graphs.from_dense(wr), graphs.from_dense(wc)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, np.ones(n), 0, 0.0, seed=n)
    w = configs.Workload(f"sync_{n}", n, p, R, C, 1, 1, 0.03, 0, "diag_quadratic",
                         problems.diag_quadratic(n, p, n), sched, 0.1, 70 + n, 1e-4)
    a, b = _pair(w)
    x0 = np.random.default_rng(n).standard_normal((n, p)).astype(np.float32)
    for g in (a, b):
        if variant:
            g.set_optimizer(0.8, 0.01)
            g.set_gamma_schedule(17, 0.5)
        g.init(x0, None)
    for steps in (40, 1, 25):
        for g in (a, b):
            g.sync_run(steps, w.gamma, None)
            g.check()
        for f_ in ("X", "Z", "G", "T_NODE", "ROUND") + (("MOMENTUM",) if variant else ()):
            assert np.array_equal(a.read(f_), b.read(f_)), (n, variant, steps, f_)
    assert np.abs(a.read("X") - x0).max() > 1e-3


def test_generated_schedules_and_events():
    w = configs.config2(p=2052, rounds=0)
    a, b = _pair(w)
    p_act = torch.full((w.n,), 0.7, dtype=torch.float32)
    for g in (a, b):
        g.init(None, None)
        g.run_generated(90, 77, p_act.to(g.device), 4, 0.1, w.gamma)
        g.check()
    _same(a, b, "generated")
    for g in (a, b):
        g.run_events(40, 78, None, 4, 0.1, w.gamma)     # one agent per iteration: always one pass per round
        g.run_generated(33, 79, p_act.to(g.device), 2, 0.0, w.gamma)
    _same(a, b, "generated after events")


def test_odd_p_runs_one_pass_per_round_and_momentum_variant_same_bits():
    """p not a multiple of four: the call must simply run one pass per round.  The optimizer variant
    (heavy-ball buffer, weight decay, step-size schedule) goes through the multi-round kernel."""
    w = configs.config2(p=1027, rounds=0)
    a, b = _pair(w)
    assert rfast_block_info(a.ctx) == 0
    for g in (a, b):
        g.init(None, None)
    st, dev = harness.upload_chunk(a, w, 0, 40)
    args = [dev[k] for k in ("active", "delay_R", "delay_C", "drop_R", "drop_C")]
    for g in (a, b):
        g.run(40, *args, w.gamma)
    _same(a, b, "odd p")
    w = configs.config2(p=1028, rounds=0)
    w.sched.p_active[:] = 0.7
    a, b = _pair(w)
    for g in (a, b):
        g.set_optimizer(0.9, 0.01)
        g.set_gamma_schedule(15, 0.5)
        g.init(None, None)
    assert rfast_block_info(a.ctx) == 4
    st, dev = harness.upload_chunk(a, w, 0, 40)
    args = [dev[k] for k in ("active", "delay_R", "delay_C", "drop_R", "drop_C")]
    for g in (a, b):
        g.run(40, *args, w.gamma)
        g.check()
    _same(a, b, "momentum")
    assert np.array_equal(a.read("MOMENTUM"), b.read("MOMENTUM"))
    assert np.abs(a.read("MOMENTUM")).max() > 0
    # weight decay alone: the variant's kernel without a heavy-ball buffer
    a, b = _pair(w)
    for g in (a, b):
        g.set_optimizer(0.0, 0.02)
        g.init(None, None)
    for g in (a, b):
        g.run(40, *[dev[k] for k in ("active", "delay_R", "delay_C", "drop_R", "drop_C")], w.gamma)
        g.check()
    _same(a, b, "weight decay")


@pytest.mark.parametrize("case", ["least_squares_full_gradient", "logistic_minibatches", "least_squares_weight_decay",
                                  "several_coordinates_per_lane", "rows_longer_than_a_wavefront_pass"])
def test_whole_problem_in_one_workgroup(case):
    """Least squares and logistic regression small enough for the LDS of one compute unit: rfast_run takes
    stretches of rounds with one launch of a single workgroup; same bits as the chain of four kernels per round
    (launches cut by the rebase interval and by the step-size schedule, a single round in between, generated
    schedules; with the objective data in LDS and without)."""
    if case == "logistic_minibatches":
        w = configs.config1(p=32, samples=96, batch=16, rounds=0)       # data stay in global memory
    elif case == "several_coordinates_per_lane":
        w = configs.config0(p=192, rounds=0)     # n p = 1536 > 1024 lanes, p / 4 = 48 and p no powers of two
    elif case == "rows_longer_than_a_wavefront_pass":
        # p / 4 = 128: two float4 per lane of the rows kernel's wavefront; 12 rows: no multiple of 4 x 4; data in LDS
        from rfast_workloads import graphs, problems
        r, c = graphs.directed_ring(3)
        w = configs._mk("ring3_least_squares_p512", 3, 512, r, c, 1, 0.01, 0, "least_squares",
                        problems.least_squares(3, 512, 12, 5), 0.6, 0.1, 5, samples=12, burst=2)
    else:
        w = configs.config0(rounds=0)                                   # data in LDS too
    a, b = _pair(w)
    assert rfast_block_info(a.ctx) != 0 and rfast_block_info(b.ctx) == 0
    rng = np.random.default_rng(3)
    x0 = (0.1 * rng.standard_normal((w.n, w.p))).astype(np.float32)
    for g in (a, b):
        rfast_set_rebase_interval(g.ctx, 29)
        if case == "least_squares_weight_decay":
            g.set_optimizer(0.0, 0.01)
        g.set_gamma_schedule(25, 0.8)
        g.init(x0, w.sched.initial_batch())
    st, dev = harness.upload_chunk(a, w, 0, 120)
    names = ("active", "delay_R", "delay_C", "drop_R", "drop_C")
    for lo, hi in ((0, 50), (50, 51), (51, 120)):
        for g in (a, b):
            bi = None if dev["batch_idx"] is None else dev["batch_idx"][lo:hi].contiguous()
            g.run(hi - lo, *[dev[k][lo:hi].contiguous() for k in names], w.gamma, bi)
            g.check()
        _same(a, b, (case, hi), INTEGER_REST)
    p_act = torch.full((w.n,), 0.6, dtype=torch.float32)
    for g in (a, b):
        g.run_generated(70, 5, p_act.to(g.device), w.sched.d_max, 0.1, w.gamma)
        g.check()
    _same(a, b, (case, "generated"), INTEGER_REST)
    assert np.abs(a.read("X") - x0).max() > 1e-3
@pytest.mark.parametrize("case", ["logistic_minibatches", "least_squares_full_gradient", "rows_longer_than_one_pass",
                                  "weight_decay_many_in_edges"])
def test_round_as_two_kernels(case):
    """Least squares and logistic regression too large for one workgroup: consecutive rounds are two kernels each
    (rows; columns + track + the mixing of the next round) instead of four; same bits.  Uploaded schedules in
    calls of several lengths (a single round runs the four kernels), then a generated one; a batch that is no
    multiple of the four wavefronts, rows of more than 4096 coordinates, more in-edges than one batch of loads,
    buffers that leave their sender's ring (losses in bursts), a step-size schedule (the mixing of the next round
    runs with the next round's step size)."""
    if case == "logistic_minibatches":
        w = configs.config1(p=512, samples=128, batch=22, rounds=0)
    elif case == "least_squares_full_gradient":
        w = configs.config0(p=2048, m=19, rounds=0)
    elif case == "rows_longer_than_one_pass":
        w = configs.config1(p=4616, samples=64, batch=9, rounds=0)       # 4096 + 520: a second, ragged pass over a row
    else:
        # a star: the root pulls from and pushes to 11 leaves (more in-edges than the eight loaded at a time)
        n = 12
        adj = np.eye(n)
        adj[0, :] = 1
        adj[:, 0] = 1
        wr = adj / adj.sum(1, keepdims=True)
        wc = adj / adj.sum(0, keepdims=True)
        w = configs._mk("star12_logistic", n, 260, wr, wc, 2, 0.05, 0, "logistic", problems.logistic(n, 260, 40, 3), 0.6,
                        0.3, 3, batch=8, samples=40, burst=3)
    if case == "least_squares_full_gradient":
        w.gamma = 0.002                      # 19 rows in 2048 dimensions: the largest curvature is about a hundred
    a, b = _pair(w)
    assert rfast_block_info(a.ctx) == 0     # no launch over several rounds here: it is the round itself that differs
    rng = np.random.default_rng(11)
    x0 = (0.1 * rng.standard_normal((w.n, w.p))).astype(np.float32)
    for g in (a, b):
        rfast_set_rebase_interval(g.ctx, 31)
        if case == "weight_decay_many_in_edges":
            g.set_optimizer(0.0, 0.01)
        g.set_gamma_schedule(20, 0.8)
        g.init(x0, w.sched.initial_batch())
    st, dev = harness.upload_chunk(a, w, 0, 80)
    names = ("active", "delay_R", "delay_C", "drop_R", "drop_C")
    for lo, hi in ((0, 45), (45, 46), (46, 80)):
        for g in (a, b):
            bi = None if dev["batch_idx"] is None else dev["batch_idx"][lo:hi].contiguous()
            g.run(hi - lo, *[dev[k][lo:hi].contiguous() for k in names], w.gamma, bi)
            g.check()
        _same(a, b, (case, hi))
    p_act = torch.full((w.n,), 0.6, dtype=torch.float32)
    for g in (a, b):
        g.run_generated(40, 5, p_act.to(g.device), w.sched.d_max, 0.1, w.gamma)
        g.check()
    _same(a, b, (case, "generated"))
    assert np.abs(a.read("X") - x0).max() > 1e-3
    assert np.isfinite(a.read("X")).all() and np.isfinite(a.read("Z")).all()
