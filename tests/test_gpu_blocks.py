"""Several rounds per launch with the per-coordinate state resident in LDS must give the same bits
as one kernel pass per round: same plans, same arithmetic, only the memory the values travel
through differs.  Uploaded and generated schedules, launches cut short by the rebase interval
and by the step-size schedule, graphs whose rings spill S4 buffers, ragged last tile."""
import numpy as np
import pytest
import torch

from paper_2307_11617_amd import rfast_use_blocks, rfast_set_rebase_interval
from rfast_workloads import configs, graphs, problems
from rfast_workloads.schedule import ScheduleSpec

import harness

pytestmark = pytest.mark.gpu
FIELDS = ("X", "Z", "G", "V_RING", "SIGMA_RING", "RHO_TILDE", "T_NODE", "TAU_R", "TAU_C", "SLOT_R", "SLOT_C", "ROUND")


def _pair(w):
    a, b = harness.make_gpu(w), harness.make_gpu(w)
    rfast_use_blocks(b.ctx, False)
    return a, b


def _same(a, b, where):
    for f in FIELDS:
        assert np.array_equal(a.read(f), b.read(f)), (where, f)


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_uploaded_schedules(seed):
    rng = np.random.default_rng(seed)
    n = [16, 5, 33, 9][seed]
    p = [1028, 64, 260, 4100][seed]
    d_max, burst = [4, 0, 2, 1][seed], [4, 1, 2, 3][seed]
    wr, wc = graphs.random_digraph(n, rng, extra=0.4) if seed else graphs.bidirectional_ring(n)
    R, C = graphs.from_dense(wr), graphs.from_dense(wc)
    p_act = np.where(np.arange(n) % 4 == 1, 0.1, 0.9)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, p_act, d_max, 0.3, seed=seed)
    w = configs.Workload(f"blocks_{seed}", n, p, R, C, d_max + burst - 1, burst, 0.02, 0, "diag_quadratic",
                         problems.diag_quadratic(n, p, seed), sched, 0.1, 50 + seed, 1e-4)
    a, b = _pair(w)
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


def test_not_taken_where_it_does_not_apply():
    """Momentum variant, p not a multiple of four: the call must simply run one pass per round."""
    w = configs.config2(p=1027, rounds=0)
    a, b = _pair(w)
    for g in (a, b):
        g.init(None, None)
    st, dev = harness.upload_chunk(a, w, 0, 20)
    args = [dev[k] for k in ("active", "delay_R", "delay_C", "drop_R", "drop_C")]
    for g in (a, b):
        g.run(20, *args, w.gamma)
    _same(a, b, "odd p")
    w = configs.config2(p=1024, rounds=0)
    a, b = _pair(w)
    for g in (a, b):
        g.set_optimizer(0.9, 0.01)
        g.init(None, None)
        g.run(20, *[v.clone() for v in args], w.gamma)
    _same(a, b, "momentum")
