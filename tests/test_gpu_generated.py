"""On-device schedule generation: the generated masks must equal the reference
generator bit for bit, and a run driven by them must stay on the oracle's
trajectory when the oracle is driven by the reference schedule."""
import numpy as np
import pytest
import torch

from oracle import schedule_gen as sg
from rfast_workloads import configs

import harness

pytestmark = pytest.mark.gpu


def _ref(w, seed, r, p_active, d_max, p_drop):
    return sg.generate_round(seed, r, w.n, w.R.nnz_off, w.C.nnz_off, p_active, d_max, p_drop, w.sched.batch, w.sched.samples)


def test_generated_schedule_is_bit_exact():
    w = configs.config1(p=128, samples=100, batch=24, rounds=0)
    gpu = harness.make_gpu(w)
    gpu.init(None, w.sched.initial_batch())
    p_act = np.linspace(0.1, 1.0, w.n).astype(np.float32)
    dev_p = torch.from_numpy(p_act).to(gpu.device)
    for r in range(6):
        gpu.run_generated(1, 12345678901234, dev_p, 5, 0.3, w.gamma)
        ref = _ref(w, 12345678901234, r, p_act, 5, 0.3)
        for name, key in (("SCHED_ACTIVE", "active"), ("SCHED_DELAY_R", "delay_R"), ("SCHED_DELAY_C", "delay_C"),
                          ("SCHED_DROP_R", "drop_R"), ("SCHED_DROP_C", "drop_C"), ("SCHED_BATCH", "batch_idx")):
            assert np.array_equal(gpu.read(name), ref[key]), (r, name)
    gpu.check()
    with pytest.raises(Exception):
        gpu.run_generated(1, 1, dev_p, w.D, 0.3, w.gamma)     # max_delay beyond D - burst + 1


@pytest.mark.parametrize("which", ["diag", "logistic"])
def test_generated_run_matches_oracle(which):
    if which == "diag":
        w = configs.config3(p=1028, rounds=0)
        d_max, p_drop = 16, 0.2
    else:
        w = configs.config1(p=132, samples=64, batch=16, rounds=0)
        d_max, p_drop = 8, 0.05
    seed = 99
    p_act = w.sched.p_active.astype(np.float32)
    orc = harness.make_oracle(w)
    gpu = harness.make_gpu(w)
    gpu.init(None, w.sched.initial_batch())
    dev_p = torch.from_numpy(p_act).to(gpu.device)
    for chunk in range(3):
        gpu.run_generated(100, seed, dev_p, d_max, p_drop, w.gamma)
        for r in range(chunk * 100, chunk * 100 + 100):
            q = _ref(w, seed, r, p_act, d_max, p_drop)
            orc.round(q["active"], q["delay_R"], q["delay_C"], q["drop_R"], q["drop_C"], w.gamma, q["batch_idx"])
        gpu.check()
        sl = orc.slots()
        assert np.array_equal(gpu.read("T_NODE"), sl["t"])
        assert np.array_equal(gpu.read("TAU_R"), sl["tau_v"]) and np.array_equal(gpu.read("TAU_C"), sl["tau_rho"])
        gn = float(np.linalg.norm(orc.g))
        ex, ez = harness.rel_l2(gpu.read("X"), orc.x), harness.rel_l2(gpu.read("Z"), orc.z, 1e-3 * gn)
        assert ex <= 1e-4 and ez <= 1e-4, (chunk, ex, ez)
    assert 0 < orc.t.min() < orc.t.max()


@pytest.mark.parametrize("which", ["diag", "logistic"])
def test_graph_replay_equals_eager_launches(which):
    """A HIP graph of 16 generated rounds, replayed several times with eager work and
    host synchronisations in between, must leave exactly the state eager launches leave."""
    import paper_2307_11617_amd as rf
    if which == "diag":
        w = configs.config2(p=2048, rounds=0)
        d_max, p_drop = 4, 0.02
    else:
        w = configs.config1(p=132, samples=64, batch=16, rounds=0)
        d_max, p_drop = 8, 0.05
    p_act = torch.full((w.n,), 0.6, dtype=torch.float32)
    eager, graph = harness.make_gpu(w), harness.make_gpu(w)
    dev_p = p_act.to(eager.device)
    for g in (eager, graph):
        g.init(None, w.sched.initial_batch())
    rf.rfast_use_graphs(graph.ctx, True)
    fields = ("X", "Z", "G", "V_RING", "SIGMA_RING", "RHO_TILDE", "T_NODE", "TAU_R", "TAU_C", "DELIV_R", "DELIV_C", "ROUND")
    for rounds in (16, 37, 5, 48, 16):          # replays, remainders, a short eager-only call
        eager.run_generated(rounds, 7, dev_p, d_max, p_drop, w.gamma)
        graph.run_generated(rounds, 7, dev_p, d_max, p_drop, w.gamma)
        graph.check()
        for f in fields:
            assert np.array_equal(eager.read(f), graph.read(f)), (rounds, f)
        graph.diagnostics()                      # unrelated eager work between replays
    # changing an argument rebuilds the graph
    eager.run_generated(32, 8, dev_p, d_max, p_drop, w.gamma * 0.5)
    graph.run_generated(32, 8, dev_p, d_max, p_drop, w.gamma * 0.5)
    for f in fields:
        assert np.array_equal(eager.read(f), graph.read(f)), f
    rf.rfast_use_graphs(graph.ctx, False)
    eager.run_generated(20, 8, dev_p, d_max, p_drop, w.gamma)
    graph.run_generated(20, 8, dev_p, d_max, p_drop, w.gamma)
    assert np.array_equal(eager.read("X"), graph.read("X"))


@pytest.mark.parametrize("which", ["diag", "logistic"])
def test_event_driven_run_is_algorithm_2_taken_literally(which):
    """One agent per global iteration, delays in global iterations: the device draws i^k,
    the oracle activates that very agent with Algorithm 2's steps (its `activate`, through
    a round whose mask is one-hot).  Stragglers are agents with small selection weights."""
    if which == "diag":
        w = configs.config3(p=1028, rounds=0)
        d_max, p_drop, weights = 16, 0.2, np.where(np.arange(w.n) % 9 == 0, 0.05, 1.0).astype(np.float32)
        w.gamma = 0.002
    else:
        w = configs.config1(p=132, samples=64, batch=16, rounds=0)
        d_max, p_drop, weights = 8, 0.05, None
    seed = 4242
    orc = harness.make_oracle(w)
    gpu = harness.make_gpu(w)
    gpu.init(None, w.sched.initial_batch())
    drawn = np.zeros(w.n, dtype=np.int64)
    for chunk in range(4):
        gpu.run_events(150, seed, weights, d_max, p_drop, w.gamma)
        for k in range(chunk * 150, chunk * 150 + 150):
            q = sg.generate_event(seed, k, w.n, w.R.nnz_off, w.C.nnz_off, weights, d_max, p_drop, w.sched.batch, w.sched.samples)
            assert q["active"].sum() == 1
            drawn += q["active"]
            orc.round(q["active"], q["delay_R"], q["delay_C"], q["drop_R"], q["drop_C"], w.gamma, q["batch_idx"])
        gpu.check()
        assert np.array_equal(gpu.read("SCHED_ACTIVE"), q["active"])       # the last iteration's draw
        sl = orc.slots()
        assert np.array_equal(gpu.read("T_NODE"), sl["t"]) and int(gpu.read("T_NODE").sum()) == (chunk + 1) * 150
        assert np.array_equal(gpu.read("TAU_R"), sl["tau_v"]) and np.array_equal(gpu.read("TAU_C"), sl["tau_rho"])
        gn = float(np.linalg.norm(orc.g))
        ex = harness.rel_l2(gpu.read("X"), orc.x)
        ez = harness.rel_l2(gpu.read("Z"), orc.z, 1e-3 * gn)
        assert ex <= w.tol and ez <= w.tol, (chunk, ex, ez)
    if weights is not None:
        assert drawn[np.arange(w.n) % 9 == 0].sum() < 0.05 * drawn.sum()    # the slow agents are rarely drawn
    with pytest.raises(Exception):
        gpu.run_events(1, seed, np.zeros(w.n, np.float32), d_max, p_drop, w.gamma)
    with pytest.raises(Exception):
        gpu.run_events(1, seed, weights, w.D, p_drop, w.gamma)
