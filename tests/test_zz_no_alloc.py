"""rfast_diagnostics_static (the entry point that allocates nothing: its scratch is a static device array of the
library) against rfast_diagnostics, through the C ABI, on calls in a row that share the one array: a larger input
first, then a smaller one, for the objective that stages the node average in the scratch and for the one that does
not."""
import numpy as np
import pytest
import torch

import paper_2307_11617_amd as rf
from rfast_workloads import configs

import harness

pytestmark = pytest.mark.gpu
KEYS = ("consensus_sq", "z_sq", "conservation_sq", "gsum_sq", "xbar_gap_sq", "loss_at_xbar")


def _advance(w, rounds):
    gpu = harness.make_gpu(w)
    gpu.init(None, w.sched.initial_batch())
    st, dev = harness.upload_chunk(gpu, w, 0, rounds)
    gpu.run(rounds, dev["active"], dev["delay_R"], dev["delay_C"], dev["drop_R"], dev["drop_C"], w.gamma, dev["batch_idx"])
    gpu.check()
    return gpu


def _both(gpu, xstar):
    want = gpu.diagnostics(xstar)
    out = torch.full((6,), float("nan"), dtype=torch.float64, device=gpu.device)
    rf.rfast_diagnostics_static(gpu.ctx, xstar, out)
    torch.cuda.synchronize()
    return want, dict(zip(KEYS, out.cpu().numpy().tolist()))


def _close(want, got, where):
    for k in KEYS:
        a, b = want[k], got[k]
        # the same fp64 partial sums, added by atomics in whatever order the workgroups finish; the conservation
        # residual is a sum of squares of fp32 rounding errors and agrees to the same relative accuracy
        assert abs(a - b) <= 1e-9 * max(abs(a), abs(b)) + 1e-300, (where, k, a, b)


@pytest.mark.parametrize("make", [lambda p: configs.config1(p=p, samples=128, batch=16, rounds=12),
                                  lambda p: configs.config2(p=p, rounds=12),
                                  lambda p: configs.config0(p=p, rounds=12)])
def test_static_scratch_matches_workspace_scratch_on_calls_in_a_row(make):
    big, small = make(4096), make(260)
    g_big, g_small = _advance(big, 12), _advance(small, 12)
    for gpu, w, tag in ((g_big, big, "larger first"), (g_small, small, "then smaller"), (g_big, big, "larger again")):
        xstar = torch.linspace(-1.0, 1.0, w.p, dtype=torch.float32, device=gpu.device)
        _close(*_both(gpu, xstar), (tag, w.name))
        want, got = _both(gpu, None)
        assert got["xbar_gap_sq"] == -1.0 and want["xbar_gap_sq"] == -1.0
        _close(want, got, (tag, w.name, "no x*"))


def test_softmax_loss_through_the_static_scratch():
    w = configs.config4(d=64, K=32, samples=128, batch=64, rounds=6)
    gpu = _advance(w, 6)
    _close(*_both(gpu, None), w.name)


def test_sizes_beyond_the_static_scratch_are_rejected():
    w = configs.config1(p=(1 << 20) + 64, samples=2, batch=1, rounds=1)
    gpu = harness.make_gpu(w)
    gpu.init(None, w.sched.initial_batch())
    out = torch.zeros(6, dtype=torch.float64, device=gpu.device)
    with pytest.raises(rf.RFastError) as err:
        rf.rfast_diagnostics_static(gpu.ctx, None, out)
    assert err.value.code == -4 and "static scratch" in str(err.value)
    gpu.diagnostics()   # the entry point with its scratch in the workspace takes the same size
