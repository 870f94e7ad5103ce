"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle on the
same seeded inputs.  Integer state bit-exact; x and z within the stated
relative-L2 tolerance at every checkpoint."""
import numpy as np
import pytest

from rfast_workloads import configs

import harness

pytestmark = pytest.mark.gpu


def _report(name, worst):
    print(f"\n[{name}] worst rel-L2: " + ", ".join(f"{k} {v:.2e}" for k, v in worst.items()), flush=True)


def test_config0_full():
    w = configs.config0()
    worst, orc, gpu = harness.run_parity(w, w.rounds, every=100)
    _report(w.name, worst)


@pytest.mark.parametrize("p", [4096 + 1024 + 8, 1003])
def test_config2_small(p):
    """Several tiles and a ragged tail (float4 path), and the scalar path (p odd)."""
    w = configs.config2(p=p, rounds=300)
    worst, orc, gpu = harness.run_parity(w, 300, every=100)
    _report(w.name + f" p={p}", worst)
    d = gpu.diagnostics()
    assert d["conservation_sq"] <= 1e-8 * max(d["gsum_sq"], 1.0)


def test_config3_small():
    w = configs.config3(p=2052, rounds=600)
    worst, orc, gpu = harness.run_parity(w, 600, every=100)
    _report(w.name, worst)


def test_config1_small():
    w = configs.config1(p=520, samples=256, batch=32, rounds=500)
    worst, orc, gpu = harness.run_parity(w, 500, every=100)
    _report(w.name, worst)


def test_config4_small():
    """bf16 MFMA softmax gradient: several row blocks and feature blocks, two class tiles."""
    w = configs.config4(d=192, K=64, samples=320, batch=128, rounds=300)
    worst, orc, gpu = harness.run_parity(w, 300, every=100)
    _report(w.name, worst)


def test_config4_small_all_classes():
    """K = 128 (four class tiles, the full-size wave layout) at a small d."""
    w = configs.config4(d=256, K=128, samples=256, batch=64, rounds=200)
    worst, orc, gpu = harness.run_parity(w, 200, every=100)
    _report(w.name + " d=256", worst)


@pytest.mark.parametrize("K", [32, 96])
def test_config4_small_other_class_counts(K):
    """K = 32: one class tile, 32 features per state tile (the mixing pass writes the bf16 copy of
    the weights itself); K = 96 does not divide the state tile, so the separate conversion pass runs."""
    w = configs.config4(d=128, K=K, samples=192, batch=64, rounds=150)
    worst, orc, gpu = harness.run_parity(w, 150, every=50)
    _report(w.name + f" K={K}", worst)


def test_x0_nonzero_and_noise_free():
    rng = np.random.default_rng(0)
    w = configs.config2(p=2048, rounds=200)
    w.noise_std = 0.0
    x0 = rng.standard_normal((w.n, w.p)).astype(np.float32)
    worst, orc, gpu = harness.run_parity(w, 200, every=50, x0=x0)
    _report(w.name + " x0!=0", worst)
