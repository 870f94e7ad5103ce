"""Parity at the full sizes of the five workloads, in the launch configuration
bench.py times.  Where the oracle cannot hold the whole state (configs 2 and 3:
p in the millions) it runs on a deterministic coordinate subset: the objective
is separable, so those coordinates evolve exactly as inside the full vector,
and the GPU's values at them are compared.  Integer state is always compared
in full."""
import os
import sys

import numpy as np
import pytest

from rfast_workloads import configs

import harness

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _coords(p, step=173):
    c = np.unique(np.concatenate([np.arange(0, p, step), np.arange(0, 64), np.arange(p - 64, p),
                                  np.arange(p // 2 - 32, p // 2 + 32)]))
    return c.astype(np.int64)


def _report(name, worst):
    print(f"\n[{name}] worst rel-L2: " + ", ".join(f"{k} {v:.2e}" for k, v in worst.items()), flush=True)


# Stride of the sampled coordinates of config 2: odd and coprime with every tile width, so that the sample
# walks through every lane of a node, every element of a float4 and every output word of the noise generator.
STRIDE2 = 1381


def test_config2_full_sampled():
    w = configs.config2()
    c = _coords(w.p, STRIDE2)
    worst, orc, gpu = harness.run_parity(w, w.rounds, every=100, coords=c, verbose=True)
    _report(w.name + f" ({c.size} sampled coordinates)", worst)


def test_config2_full_sampled_in_the_launches_of_the_benchmark():
    """bench.py's default: 12 warm-up rounds, then the 500 rounds of the workload as one call, which is one
    launch of the multi-round kernel ending at round 512 (where the automatic rebase falls due)."""
    w = configs.config2()
    c = _coords(w.p, STRIDE2)
    assert len({int(k) % 64 for k in c}) == 64
    worst, orc, gpu = harness.run_parity(w, 512, every=[12, 500], coords=c, verbose=True)
    _report(w.name + f" ({c.size} sampled coordinates, calls of 12 and 500 rounds)", worst)


def test_config3_full_sampled():
    w = configs.config3()
    c = _coords(w.p, 173)
    worst, orc, gpu = harness.run_parity(w, w.rounds, every=100, coords=c, verbose=True)
    _report(w.name + f" ({c.size} sampled coordinates)", worst)


def test_config2_in_the_launches_of_a_short_benchmark_run():
    """`bench.py --steps 20 --warmup 5`: 5 rounds one pass each, then launches of 20 rounds."""
    w = configs.config2(rounds=65)
    c = _coords(w.p, STRIDE2)
    worst, orc, gpu = harness.run_parity(w, 65, every=[5, 20, 20, 20], coords=c, verbose=True)
    _report(w.name + f" ({c.size} sampled coordinates, calls of 5, 20, 20, 20 rounds)", worst)


def test_config1_full():
    w = configs.config1()
    # the library's defaults, automatic rebase every 512 rounds included (the rings are compared in the small case)
    worst, orc, gpu = harness.run_parity(w, w.rounds, every=100, verbose=True, check_rings=False)
    _report(w.name + f" ({w.rounds} rounds)", worst)


def test_config4_first_rounds_against_the_live_oracle():
    w = configs.config4()
    worst, orc, gpu = harness.run_parity(w, 200, every=100, verbose=True, check_rings=False)
    _report(w.name + " (200 rounds)", worst)


def test_config4_full_size():
    """All 3000 rounds against the oracle's stored checkpoints (tests/golden/make_checkpoints.py wrote them
    from the fp64 oracle alone, which needs about 0.2 s per round): integer state in full, x and z on the
    stored coordinate sample, and of the full vectors the per-node norms and eight +-1 projections."""
    sys.path.insert(0, GOLDEN)
    from make_checkpoints import projection_signs
    ck = np.load(os.path.join(GOLDEN, "cfg4_checkpoints.npz"))
    w = configs.config4()
    assert str(ck["workload"]) == w.name and int(ck["round"][-1]) == w.rounds
    coords = ck["coords"]
    signs = projection_signs(w.p).astype(np.float64)
    gpu = harness.make_gpu(w)
    gpu.init(None, w.sched.initial_batch())
    tol, worst = w.tol, {"x": 0.0, "z": 0.0}
    r0 = 0
    for q, r1 in enumerate(int(r) for r in ck["round"]):
        st, dev = harness.upload_chunk(gpu, w, r0, r1)
        gpu.run(r1 - r0, dev["active"], dev["delay_R"], dev["delay_C"], dev["drop_R"], dev["drop_C"], w.gamma, dev["batch_idx"])
        gpu.check()
        assert np.array_equal(gpu.read("T_NODE"), ck["t"][q]), f"t differs at round {r1}"
        assert np.array_equal(gpu.read("TAU_R"), ck["tau_v"][q]), f"tau_v differs at round {r1}"
        assert np.array_equal(gpu.read("TAU_C"), ck["tau_rho"][q]), f"tau_rho differs at round {r1}"
        x, z = gpu.read("X").astype(np.float64), gpu.read("Z").astype(np.float64)
        gn = float(np.linalg.norm(ck["g_norm"][q]))
        ex = harness.rel_l2(x[:, coords], ck["x_s"][q].astype(np.float64))
        ez = harness.rel_l2(z[:, coords], ck["z_s"][q].astype(np.float64), 1e-3 * gn * np.sqrt(len(coords) / w.p))
        worst = {"x": max(worst["x"], ex), "z": max(worst["z"], ez)}
        print(f"round {r1}: rel-L2 on the sample x {ex:.2e} z {ez:.2e}", flush=True)
        assert ex <= tol and ez <= tol, f"round {r1}: x {ex:.3e} z {ez:.3e} (tol {tol})"
        for name, got, norm, proj in (("x", x, ck["x_norm"][q], ck["x_proj"][q]), ("z", z, ck["z_norm"][q], ck["z_proj"][q])):
            floor = 1e-3 * ck["g_norm"][q] if name == "z" else 0.0
            scale = np.maximum(norm, floor)
            assert (np.abs(np.linalg.norm(got, axis=1) - norm) <= tol * scale).all(), f"round {r1}: norm of {name}"
            # an error e of norm <= tol ||ref|| moves a +-1 projection by about ||e||; six standard deviations
            assert (np.abs(got @ signs.T - proj) <= 6.0 * tol * scale[:, None]).all(), f"round {r1}: projections of {name}"
        r0 = r1
    _report(w.name + f" ({w.rounds} rounds, stored oracle checkpoints)", worst)
