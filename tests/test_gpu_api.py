"""GPU tests of the ABI's behaviour around the round itself: diagnostics against
the oracle's, device-side range checks (inputs are clamped, never faulting),
single rounds vs stacked runs, re-initialisation, the profiling hooks."""
import numpy as np
import pytest
import torch

import paper_2307_11617_amd as rf
from rfast_workloads import configs

import harness

pytestmark = pytest.mark.gpu


def _dev_round(gpu, q):
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(gpu.device)
    return t(q.active), t(q.delay_R), t(q.delay_C), t(q.drop_R), t(q.drop_C), t(q.batch_idx)


def test_diagnostics_match_oracle():
    w = configs.config3(p=4100, rounds=150)
    worst, orc, gpu = harness.run_parity(w, 150, every=50)
    h, c = w.data["h"].astype(np.float64), w.data["c"].astype(np.float64)
    x_star = (h * c).sum(axis=0) / h.sum(axis=0)
    ref = orc.diagnostics(x_star)
    got = gpu.diagnostics(torch.from_numpy(x_star.astype(np.float32)).to(gpu.device))
    for key in ("consensus_sq", "z_sq", "gsum_sq", "xbar_gap_sq", "loss_at_xbar"):
        assert abs(got[key] - ref[key]) <= 2e-4 * abs(ref[key]), (key, got[key], ref[key])
    # Lemma 3 in fp32: the residual is rounding noise relative to the tracked mass
    assert got["conservation_sq"] <= 1e-9 * (got["gsum_sq"] + got["z_sq"])
    assert gpu.diagnostics(None)["xbar_gap_sq"] == -1.0


def test_diagnostics_near_consensus():
    """Nodes that agree to a few units in the last place of large values: the consensus error is the sum of squared
    deviations from the mean, a quantity 1e-14 of the squared values; computed in one walk over the nodes it must
    not be lost to cancellation.  Expected value from the same fp32 numbers in NumPy fp64 (the definition)."""
    w = configs.config2(p=4100, rounds=5)
    gpu = harness.make_gpu(w)
    gpu.init()
    rng = np.random.default_rng(5)
    base = rng.normal(100.0, 30.0, size=w.p).astype(np.float32)
    x = np.stack([np.nextafter(base, np.float32(np.inf)) if i % 3 == 0 else base for i in range(w.n)]).astype(np.float32)
    x[1] = np.nextafter(np.nextafter(base, np.float32(-np.inf)), np.float32(-np.inf))
    gpu.write("X", x)
    x64 = x.astype(np.float64)
    xbar = x64.mean(axis=0)
    want = float(((x64 - xbar) ** 2).sum())
    got = gpu.diagnostics()
    assert want > 0 and abs(got["consensus_sq"] - want) <= 1e-9 * want, (got["consensus_sq"], want)
    c, h = w.data["c"].astype(np.float64), w.data["h"].astype(np.float64)
    loss = float((0.5 * h * (xbar - c) ** 2).sum())
    assert abs(got["loss_at_xbar"] - loss) <= 1e-12 * loss, (got["loss_at_xbar"], loss)


@pytest.mark.parametrize("which", ["least_squares", "logistic", "softmax"])
def test_training_loss_at_the_average_matches_oracle(which):
    """sum_i f_i(xbar) over every node's full local data, for the objectives with per-sample losses."""
    if which == "least_squares":
        w, rounds, tol = configs.config0(rounds=200), 200, 1e-5
    elif which == "logistic":
        w, rounds, tol = configs.config1(p=260, samples=96, batch=16, rounds=150), 150, 1e-5
    else:
        w, rounds, tol = configs.config4(d=128, K=64, samples=192, batch=64, rounds=100), 100, 2e-3
    worst, orc, gpu = harness.run_parity(w, rounds, every=50)
    ref = orc.diagnostics()
    got = gpu.diagnostics()
    assert abs(got["loss_at_xbar"] - ref["loss_at_xbar"]) <= tol * abs(ref["loss_at_xbar"]), (got, ref)
    for key in ("consensus_sq", "z_sq", "gsum_sq"):
        assert abs(got[key] - ref[key]) <= 1e-3 * abs(ref[key]) + 1e-12, (key, got[key], ref[key])


def test_single_rounds_equal_stacked_run():
    w = configs.config0(rounds=40)
    a, b = harness.make_gpu(w), harness.make_gpu(w)
    a.init()
    b.init()
    st, dev = harness.upload_chunk(a, w, 0, 40)
    a.run(40, dev["active"], dev["delay_R"], dev["delay_C"], dev["drop_R"], dev["drop_C"], w.gamma)
    for r in range(40):
        act, dR, dC, xR, xC, _ = _dev_round(b, w.sched.round(r))
        b.round(act, dR, dC, xR, xC, w.gamma)
    for f in ("X", "Z", "G", "V_RING", "RHO_RING", "RHO_TILDE", "T_NODE", "TAU_R", "TAU_C"):
        assert np.array_equal(a.read(f), b.read(f)), f
    # re-initialising restores the start state exactly
    g1 = a.read("G")
    a.init()
    b.init()
    assert int(a.read("ROUND")[0]) == 0 and not a.read("T_NODE").any() and not a.read("V_RING").any()
    assert np.array_equal(a.read("Z"), a.read("G")) and not np.array_equal(a.read("G"), g1)


def test_out_of_range_delay_is_clamped_and_reported():
    w = configs.config0(rounds=5)
    gpu = harness.make_gpu(w)
    gpu.init()
    q = w.sched.round(0)
    q.active[:] = 1
    q.delay_C[3] = w.D + 5
    act, dR, dC, xR, xC, _ = _dev_round(gpu, q)
    gpu.round(act, dR, dC, xR, xC, w.gamma)
    with pytest.raises(rf.RFastError) as ei:
        gpu.check()
    assert ei.value.code == -4 and "C edge 3" in str(ei.value) and "round 0" in str(ei.value)
    assert np.isfinite(gpu.read("X")).all()
    gpu.init()          # clears the sticky status
    gpu.check()


def test_out_of_range_sample_row_is_clamped_and_reported():
    w = configs.config1(p=256, samples=64, batch=16, rounds=3)
    gpu = harness.make_gpu(w)
    gpu.init(None, w.sched.initial_batch())
    q = w.sched.round(0)
    q.active[:] = 1
    q.batch_idx[5, 2] = 64
    act, dR, dC, xR, xC, bi = _dev_round(gpu, q)
    gpu.round(act, dR, dC, xR, xC, w.gamma, bi)
    with pytest.raises(rf.RFastError) as ei:
        gpu.check()
    assert ei.value.code == -4 and "node 5" in str(ei.value) and "round 0" in str(ei.value)
    assert np.isfinite(gpu.read("X")).all()


def test_out_of_range_delay_in_a_run_that_resolves_its_own_rounds():
    """Config 0 runs as one workgroup whose last wavefronts are the resolver: the same clamp and the same report."""
    w = configs.config0(rounds=6)
    gpu = harness.make_gpu(w)
    assert rf.rfast_block_info(gpu.ctx) != 0
    gpu.init()
    st, dev = harness.upload_chunk(gpu, w, 0, 6)
    assert st["active"][4].any()
    dC = dev["delay_C"].clone()
    dC[4, :] = w.D + 5            # every C edge of round 4: whichever has an active receiver is reported
    gpu.run(6, dev["active"], dev["delay_R"], dC, dev["drop_R"], dev["drop_C"], w.gamma, None)
    with pytest.raises(rf.RFastError) as ei:
        gpu.check()
    assert ei.value.code == -4 and "C edge" in str(ei.value) and "round 4" in str(ei.value), str(ei.value)
    assert np.isfinite(gpu.read("X")).all() and np.isfinite(gpu.read("Z")).all()
    # the clamped run is the run with the largest delay allowed
    ref = harness.make_gpu(w)
    ref.init()
    dC2 = dev["delay_C"].clone()
    dC2[4, :] = w.sched.d_max
    ref.run(6, dev["active"], dev["delay_R"], dC2, dev["drop_R"], dev["drop_C"], w.gamma, None)
    ref.check()
    for f in ("X", "Z", "T_NODE", "TAU_R", "TAU_C"):
        assert np.array_equal(gpu.read(f), ref.read(f)), f


@pytest.mark.parametrize("path", ["two kernels per round", "one workgroup"])
def test_out_of_range_sample_row_in_a_later_round_of_a_run(path):
    """The same report from the kernels that rfast_run uses for stretches of rounds: the round is named by its number
    (counted from rfast_init, from zero), the row is clamped."""
    w = configs.config1(p=256, samples=64, batch=16, rounds=6) if path == "two kernels per round" else \
        configs.config1(p=32, samples=96, batch=16, rounds=6)
    gpu = harness.make_gpu(w)
    assert (rf.rfast_block_info(gpu.ctx) != 0) == (path == "one workgroup")
    gpu.init(None, w.sched.initial_batch())
    st, dev = harness.upload_chunk(gpu, w, 0, 6)
    assert st["active"][4, 5]           # node 5 is active in round 4 of this seed
    bi = dev["batch_idx"].clone()
    bi[4, 5, 2] = w.sched.samples + 3
    gpu.run(6, dev["active"], dev["delay_R"], dev["delay_C"], dev["drop_R"], dev["drop_C"], w.gamma, bi)
    with pytest.raises(rf.RFastError) as ei:
        gpu.check()
    assert ei.value.code == -4 and "node 5" in str(ei.value) and "round 4" in str(ei.value), str(ei.value)
    assert np.isfinite(gpu.read("X")).all() and np.isfinite(gpu.read("Z")).all()


def test_out_of_range_class_label_is_clamped_and_reported():
    w = configs.config4(d=64, K=32, samples=128, batch=64, rounds=2)
    w.data["labels"][7, :] = 32          # one past the last class, in every sample of node 7
    gpu = harness.make_gpu(w)
    gpu.init(None, w.sched.initial_batch())
    with pytest.raises(rf.RFastError) as ei:
        gpu.check()
    assert ei.value.code == -4 and "label" in str(ei.value) and "node 7" in str(ei.value)
    assert np.isfinite(gpu.read("G")).all()


def test_binding_rejects_wrong_schedule_shapes():
    w = configs.config0(rounds=2)
    gpu = harness.make_gpu(w)
    gpu.init()
    act, dR, dC, xR, xC, _ = _dev_round(gpu, w.sched.round(0))
    with pytest.raises(rf.RFastError):
        gpu.round(act[:-1].contiguous(), dR, dC, xR, xC, w.gamma)
    with pytest.raises(rf.RFastError):
        gpu.round(act, dR.to(torch.int64), dC, xR, xC, w.gamma)
    with pytest.raises(rf.RFastError):
        gpu.round(act, dR, dC, xR, xC.cpu(), w.gamma)


def test_empty_round_and_no_edges():
    """A round with no active node changes nothing; a single isolated node works (no edges at all)."""
    w = configs.config2(p=1024, rounds=3)
    gpu = harness.make_gpu(w)
    gpu.init()
    x0, z0 = gpu.read("X"), gpu.read("Z")
    q = w.sched.round(0)
    q.active[:] = 0
    act, dR, dC, xR, xC, _ = _dev_round(gpu, q)
    gpu.round(act, dR, dC, xR, xC, w.gamma)
    gpu.check()
    assert np.array_equal(gpu.read("X"), x0) and np.array_equal(gpu.read("Z"), z0)
    assert not gpu.read("T_NODE").any() and int(gpu.read("ROUND")[0]) == 1
    # n = 1: x' = v, z' = z_half = z + g' - g
    one = (np.array([0, 1], np.int32), np.array([0], np.int32), np.array([1.0], np.float32))
    h = torch.full((1, 8), 2.0)
    c = torch.full((1, 8), 3.0)
    solo = rf.RFast(1, 8, one, one, 0, 1, "diag_quadratic", h, c)
    solo.init()
    e = torch.empty(0, dtype=torch.int32, device=solo.device)
    e8 = torch.empty(0, dtype=torch.uint8, device=solo.device)
    for _ in range(200):
        solo.round(torch.ones(1, dtype=torch.uint8, device=solo.device), e, e, e8, e8, 0.1)
    solo.check()
    np.testing.assert_allclose(solo.read("X"), 3.0, atol=1e-5)
    assert int(solo.read("T_NODE")[0]) == 200


def test_checkpoint_resume_is_bit_exact():
    """Read every field after 60 rounds, restore into a fresh context, continue both: identical bits."""
    w = configs.config3(p=1028, rounds=120)
    a = harness.make_gpu(w)
    a.init()
    st, dev = harness.upload_chunk(a, w, 0, 120)
    part = lambda g, lo, hi: g.run(hi - lo, dev["active"][lo:hi].contiguous(), dev["delay_R"][lo:hi].contiguous(),
                                   dev["delay_C"][lo:hi].contiguous(), dev["drop_R"][lo:hi].contiguous(),
                                   dev["drop_C"][lo:hi].contiguous(), w.gamma)
    part(a, 0, 60)
    ck = a.checkpoint()
    b = harness.make_gpu(w)
    b.init()
    b.restore(ck)
    part(a, 60, 120)
    part(b, 60, 120)
    a.check()
    b.check()
    for f in a.CHECKPOINT_FIELDS + ("RHO_RING",):
        assert np.array_equal(a.read(f), b.read(f)), f
    assert int(b.read("ROUND")[0]) == 120
    with pytest.raises(rf.RFastError):
        b.write("RHO_RING", a.read("RHO_RING"))


def test_rebase_keeps_long_runs_accurate():
    """The running sums grow without bound and only rho - rho~ matters; rebasing every 100
    rounds must leave the trajectory on the oracle's and reduce the fp32 error of z."""
    w = configs.config2(p=1024, rounds=3000)
    plain, _, _ = harness.run_parity(w, 3000, every=100, tol=1e-3)
    based, orc, gpu = harness.run_parity(w, 3000, every=100, tol=1e-4, rebase=True)
    print(f"\nworst rel-L2 over 3000 rounds: plain {plain}, rebased {based}")
    assert based["z"] < 0.5 * plain["z"]
    d = gpu.diagnostics()
    # fp32 rounding is never given back to the tracker, so the residual random-walks with the
    # number of rounds; after 3000 rounds it must still be far below the tracked mass
    assert d["conservation_sq"] <= 1e-6 * max(d["gsum_sq"], d["z_sq"], 1.0)
    sig = gpu.read("SIGMA_RING")
    t = gpu.read("T_NODE")
    for j in range(w.n):
        assert not sig[j, t[j] % (w.D + 2)].any()      # the latest running sum is the new origin


def test_automatic_rebase_interval_equals_manual_calls():
    w = configs.config2(p=516, rounds=300)
    a, b = harness.make_gpu(w), harness.make_gpu(w)
    a.init()
    b.init()
    rf.rfast_set_rebase_interval(b.ctx, 100)
    st, dev = harness.upload_chunk(a, w, 0, 300)
    args = lambda lo, hi: (hi - lo, dev["active"][lo:hi].contiguous(), dev["delay_R"][lo:hi].contiguous(),
                           dev["delay_C"][lo:hi].contiguous(), dev["drop_R"][lo:hi].contiguous(),
                           dev["drop_C"][lo:hi].contiguous(), w.gamma)
    for lo in (0, 100, 200):
        a.run(*args(lo, lo + 100))
        a.rebase()
    b.run(*args(0, 300))
    for f in ("X", "Z", "G", "SIGMA_RING", "RHO_TILDE", "T_NODE"):
        assert np.array_equal(a.read(f), b.read(f)), f


def test_profiling_hooks_count_launches():
    w = configs.config1(p=256, samples=64, batch=16, rounds=20)
    gpu = harness.make_gpu(w)
    gpu.init(None, w.sched.initial_batch())
    rf.rfast_profile_enable(gpu.ctx, True)
    st, dev = harness.upload_chunk(gpu, w, 0, 10)
    gpu.run(10, dev["active"], dev["delay_R"], dev["delay_C"], dev["drop_R"], dev["drop_C"], w.gamma, dev["batch_idx"])
    ms_s, n_s = rf.rfast_kernel_time(gpu.ctx, 0)
    ms_g, n_g = rf.rfast_kernel_time(gpu.ctx, 1)
    ms_r, n_r = rf.rfast_kernel_time(gpu.ctx, 2)
    # consecutive rounds of this objective are two kernels each (rows; columns + track + the next round's mixing) after
    # one mixing pass for the first; the resolver takes the ten rounds in one launch
    assert (n_s, n_g, n_r) == (11, 10, 1) and ms_s > 0 and ms_g > 0 and ms_r > 0
    # with rfast_use_blocks off: two state passes and one gradient (two kernels) per round
    rf.rfast_use_blocks(gpu.ctx, False)
    rf.rfast_profile_enable(gpu.ctx, True)
    st, dev = harness.upload_chunk(gpu, w, 10, 20)
    gpu.run(10, dev["active"], dev["delay_R"], dev["delay_C"], dev["drop_R"], dev["drop_C"], w.gamma, dev["batch_idx"])
    assert [rf.rfast_kernel_time(gpu.ctx, q)[1] for q in (0, 1, 2)] == [20, 10, 1]
    rf.rfast_profile_enable(gpu.ctx, False)
