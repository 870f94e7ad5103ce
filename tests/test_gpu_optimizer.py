"""GPU parity of the labelled optimizer variant (heavy-ball buffer on the
tracked direction, weight decay inside the sampled gradient, step-decayed step
size) against the fp64 oracle, on every objective and kernel path, plus the
entry points' own rules (init must follow, ranges, checkpoint, graph replay)."""
import numpy as np
import pytest
import torch

from rfast_workloads import configs, graphs, problems
from rfast_workloads.schedule import ScheduleSpec

import harness
from test_gpu_push_pull import _run as run_push_pull

pytestmark = pytest.mark.gpu


def _random(n, p, seed, gamma=0.02, noise=0.05):
    rng = np.random.default_rng(seed)
    wr, wc = graphs.random_digraph(n, rng, extra=0.5)
    R, C = graphs.from_dense(wr), graphs.from_dense(wc)
    sched = ScheduleSpec(n, R.nnz_off, C.nnz_off, np.full(n, 0.6), 3, 0.2, seed=seed)
    return configs.Workload(f"opt_random_n{n}_p{p}", n, p, R, C, 3 + 2, 3, gamma, 0, "diag_quadratic",
                            problems.diag_quadratic(n, p, seed), sched, noise, 99 + seed, 1e-4)


@pytest.mark.parametrize("p", [2052, 259])
def test_fused_path_momentum_decay_and_schedule(p):
    """Diagonal quadratic (one fused kernel): float4 path with a ragged tail, and the scalar path."""
    w = _random(11, p, seed=3)
    worst, orc, gpu = harness.run_parity(w, 240, every=60, momentum=0.8, weight_decay=0.05, gamma_schedule=(50, 0.5))
    print(f"\n[{w.name}] worst {worst}")
    d, ref = gpu.diagnostics(), orc.diagnostics()
    assert abs(d["loss_at_xbar"] - ref["loss_at_xbar"]) <= 1e-4 * abs(ref["loss_at_xbar"])
    assert d["conservation_sq"] <= 1e-8 * max(d["gsum_sq"], 1.0)


def test_streaming_path_on_coordinate_subset():
    """State far above the cache size (non-temporal path); the oracle follows every 4099th coordinate."""
    w = configs.config2(p=1_048_576, rounds=0)
    coords = np.unique(np.concatenate([np.arange(0, w.p, 4099), [w.p - 1]]))
    worst, orc, gpu = harness.run_parity(w, 120, every=40, coords=coords, momentum=0.9, weight_decay=1e-4,
                                         gamma_schedule=(30, 0.1), check_rings=False)
    print(f"\n[{w.name} p=2^20] worst {worst}")


def test_least_squares_full_gradient():
    w = configs.config0(rounds=0)
    worst, orc, gpu = harness.run_parity(w, 400, every=100, momentum=0.5, weight_decay=0.02)
    print(f"\n[{w.name}] worst {worst}")


def test_logistic_minibatch():
    w = configs.config1(p=520, samples=256, batch=32, rounds=0)
    worst, orc, gpu = harness.run_parity(w, 300, every=100, momentum=0.9, weight_decay=1e-3, gamma_schedule=(120, 0.1))
    print(f"\n[{w.name}] worst {worst}")


def test_softmax_bf16():
    w = configs.config4(d=192, K=64, samples=320, batch=128, rounds=0)
    worst, orc, gpu = harness.run_parity(w, 200, every=100, momentum=0.9, weight_decay=1e-2)
    print(f"\n[{w.name}] worst {worst}")


def test_push_pull_with_variant():
    w = configs.config2(p=4100, rounds=0)
    w.gamma = 0.02
    x0 = np.random.default_rng(0).standard_normal((w.n, w.p)).astype(np.float32)
    worst, orc, gpu = run_push_pull(w, 150, 50, x0=x0, momentum=0.7, weight_decay=0.05)
    print(f"\n[push-pull variant {w.name}] worst {worst}")


def test_entry_point_rules_and_checkpoint():
    from paper_2307_11617_amd import RFastError, rfast_set_optimizer
    w = _random(7, 516, seed=5)
    gpu = harness.make_gpu(w)
    gpu.init(None, None)
    with pytest.raises(RFastError):
        rfast_set_optimizer(gpu.ctx, 0.5, 0.0, None)          # momentum without a buffer
    with pytest.raises(RFastError):
        gpu.set_optimizer(1.0, 0.0)                            # momentum outside [0, 1)
    with pytest.raises(RFastError):
        gpu.set_optimizer(0.0, -1.0)
    with pytest.raises(RFastError):
        gpu.set_gamma_schedule(10, 0.0)
    with pytest.raises(RFastError):
        gpu.read("MOMENTUM")                                   # no buffer was given yet
    gpu.set_optimizer(0.9, 0.01)
    st, dev = harness.upload_chunk(gpu, w, 0, 40)
    args = lambda a, b: [dev[k][a:b] for k in ("active", "delay_R", "delay_C", "drop_R", "drop_C")]
    with pytest.raises(RFastError):                            # init has to follow set_optimizer
        gpu.run(1, *args(0, 1), w.gamma)
    gpu.init(None, None)
    gpu.set_gamma_schedule(16, 0.5)
    gpu.run(20, *args(0, 20), w.gamma)
    ck = gpu.checkpoint()
    assert "MOMENTUM" in ck and np.abs(ck["MOMENTUM"]).max() > 0
    gpu.run(20, *args(20, 40), w.gamma)
    end = {f: gpu.read(f) for f in ("X", "Z", "MOMENTUM")}
    # a second context restored from the checkpoint (round counter included: it drives the schedule) lands on the same bits
    other = harness.make_gpu(w)
    other.set_optimizer(0.9, 0.01)
    other.set_gamma_schedule(16, 0.5)
    other.init(None, None)
    other.restore(ck)
    other.run(20, *args(20, 40), w.gamma)
    for f, v in end.items():
        assert np.array_equal(other.read(f), v), f
    # zero hyper-parameters are the plain method bit for bit
    plain, zero = harness.make_gpu(w), harness.make_gpu(w)
    zero.set_optimizer(0.0, 0.0)
    for g in (plain, zero):
        g.init(None, None)
        g.run(40, *args(0, 40), w.gamma)
    assert np.array_equal(plain.read("X"), zero.read("X")) and np.array_equal(plain.read("Z"), zero.read("Z"))


def test_generated_run_with_schedule_matches_graph_replay():
    """The step size is baked into a captured graph: replays must stop at every decay
    step.  40-round decay steps are not a multiple of the 16 rounds one graph holds."""
    w = _random(9, 1028, seed=6)
    p_act = torch.full((w.n,), 0.6, dtype=torch.float32)
    out = []
    for graphs_on in (False, True):
        gpu = harness.make_gpu(w)
        gpu.set_optimizer(0.9, 1e-3)
        gpu.set_gamma_schedule(40, 0.5)
        gpu.init(None, None)
        if graphs_on:
            from paper_2307_11617_amd import rfast_use_graphs
            rfast_use_graphs(gpu.ctx, True)
        gpu.run_generated(150, 1234, p_act.to(gpu.device), 3, 0.2, 0.04)
        gpu.check()
        out.append((gpu.read("X"), gpu.read("Z"), gpu.read("MOMENTUM"), int(gpu.read("ROUND")[0])))
    assert out[0][3] == out[1][3] == 150
    for a, b in zip(out[0][:3], out[1][:3]):
        assert np.array_equal(a, b)
