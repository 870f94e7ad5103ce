"""GPU parity of the synchronous push-pull step (eq. (2) of the paper) against
its dense fp64 oracle, on the objectives and graphs of the asynchronous tests."""
import numpy as np
import pytest
import torch

from oracle import objectives as ob
from oracle.push_pull import PushPullOracle
from rfast_workloads import configs

import harness

pytestmark = pytest.mark.gpu


def _objective(w):
    d = w.data
    if w.objective == "diag_quadratic":
        return ob.DiagQuadratic(d["h"], d["c"], w.noise_std, w.noise_seed)
    if w.objective == "least_squares":
        return ob.LeastSquares(d["A"], d["b"])
    return ob.Logistic(d["X"], d["y"])


def _run(w, steps, every, x0=None, tol_g=1e-4, z_floor=1e-3, tol_z=1e-4, momentum=0.0, weight_decay=0.0):
    b0 = w.sched.initial_batch()
    orc = PushPullOracle(w.R.dense(), w.C.dense(), _objective(w), x0=x0 if x0 is not None else np.zeros((w.n, w.p)),
                         batch0=b0, momentum=momentum, weight_decay=weight_decay)
    gpu = harness.make_gpu(w)
    if momentum != 0.0 or weight_decay != 0.0:
        gpu.set_optimizer(momentum, weight_decay)
    gpu.init(x0, b0)
    worst = {"x": 0.0, "z": 0.0}
    for r0 in range(0, steps, every):
        bi = None
        if w.sched.batch > 0:
            bi = np.stack([w.sched.round(r).batch_idx for r in range(r0, r0 + every)])
        gpu.sync_run(every, w.gamma, None if bi is None else torch.from_numpy(bi).to(gpu.device))
        for k in range(every):
            orc.step(w.gamma, None if bi is None else bi[k])
        gpu.check()
        assert gpu.read("T_NODE").tolist() == [orc.t] * w.n and int(gpu.read("ROUND")[0]) == orc.t
        gn = float(np.linalg.norm(orc.g))
        ex = harness.rel_l2(gpu.read("X"), orc.x)
        ez = harness.rel_l2(gpu.read("Z"), orc.z, z_floor * gn)
        eg = harness.rel_l2(gpu.read("G"), orc.g)
        worst = {"x": max(worst["x"], ex), "z": max(worst["z"], ez)}
        assert ex <= 1e-4 and ez <= tol_z and eg <= tol_g, (r0 + every, ex, ez, eg)
        if momentum != 0.0:
            assert harness.rel_l2(gpu.read("MOMENTUM"), orc.m, z_floor * gn) <= tol_z
    return worst, orc, gpu


def test_push_pull_diag_quadratic_with_noise():
    w = configs.config2(p=4100, rounds=0)
    worst, orc, gpu = _run(w, 150, 50, x0=np.random.default_rng(0).standard_normal((w.n, w.p)).astype(np.float32))
    print(f"\n[push-pull {w.name}] worst {worst}")
    d = gpu.diagnostics()
    assert d["consensus_sq"] < 1e-2 * w.p


def test_push_pull_scalar_path_and_odd_steps():
    w = configs.config3(p=1001, rounds=0)
    w.gamma = 0.002
    worst, orc, gpu = _run(w, 75, 25)
    print(f"\n[push-pull {w.name}] worst {worst}")


def test_push_pull_least_squares_reaches_closed_form_optimum():
    w = configs.config0(p=16, m=24, rounds=0)
    w.gamma = 0.008
    # run to convergence: z -> 0 while the fp32 rounding of every g' - g stays in the tracker for
    # good (nothing restores the conserved sum), so z is compared on the scale of the gradients;
    # the same recursion in NumPy float32 is 1e-4 |g| off the fp64 one after 3000 steps
    worst, orc, gpu = _run(w, 3000, 500, tol_g=1e-3, z_floor=1.0, tol_z=4e-4)
    A, b = w.data["A"].astype(np.float64), w.data["b"].astype(np.float64)
    x_star = np.linalg.solve(sum(A[i].T @ A[i] for i in range(w.n)), sum(A[i].T @ b[i] for i in range(w.n)))
    gap = float(np.abs(gpu.read("X") - x_star).max())
    print(f"\n[push-pull {w.name}] worst {worst}, gap to x* {gap:.2e}")
    assert gap < 1e-4


def test_push_pull_logistic_minibatches():
    w = configs.config1(p=260, samples=128, batch=16, rounds=0)
    worst, orc, gpu = _run(w, 200, 50)
    print(f"\n[push-pull {w.name}] worst {worst}")


def test_async_rounds_after_reinit_are_unaffected():
    """The synchronous step borrows ring slots 0 and 1; rfast_init makes the context async-clean again."""
    w = configs.config2(p=1024, rounds=60)
    gpu = harness.make_gpu(w)
    gpu.init()
    gpu.sync_run(7, w.gamma)
    ref = harness.make_gpu(w)
    ref.init()
    gpu.init()
    st, dev = harness.upload_chunk(gpu, w, 0, 60)
    for g in (gpu, ref):
        g.run(60, dev["active"], dev["delay_R"], dev["delay_C"], dev["drop_R"], dev["drop_C"], w.gamma)
    for f in ("X", "Z", "G", "V_RING", "SIGMA_RING", "RHO_TILDE"):
        assert np.array_equal(gpu.read(f), ref.read(f)), f
