"""Parity at the full sizes of the five workloads, in the launch configuration
bench.py times.  Where the oracle cannot hold the whole state (configs 2 and 3:
p in the millions) it runs on a deterministic coordinate subset: the objective
is separable, so those coordinates evolve exactly as inside the full vector,
and the GPU's values at them are compared.  Integer state is always compared
in full."""
import os

import numpy as np
import pytest

from rfast_workloads import configs

import harness

pytestmark = pytest.mark.gpu
LONG = os.environ.get("RFAST_LONG_TESTS", "0") == "1"


def _coords(p, step=173):
    c = np.unique(np.concatenate([np.arange(0, p, step), np.arange(0, 64), np.arange(p - 64, p),
                                  np.arange(p // 2 - 32, p // 2 + 32)]))
    return c.astype(np.int64)


def _report(name, worst):
    print(f"\n[{name}] worst rel-L2: " + ", ".join(f"{k} {v:.2e}" for k, v in worst.items()), flush=True)


def test_config2_full_sampled():
    w = configs.config2()
    c = _coords(w.p, 173 * 8)
    worst, orc, gpu = harness.run_parity(w, w.rounds, every=100, coords=c, verbose=True)
    _report(w.name + f" ({c.size} sampled coordinates)", worst)


def test_config2_full_sampled_in_the_launches_of_the_benchmark():
    """bench.py's default: 12 warm-up rounds, then the 500 rounds of the workload as one call, which is one
    launch of the multi-round kernel ending at round 512 (where the automatic rebase falls due)."""
    w = configs.config2()
    c = _coords(w.p, 173 * 8)
    worst, orc, gpu = harness.run_parity(w, 512, every=[12, 500], coords=c, verbose=True)
    _report(w.name + f" ({c.size} sampled coordinates, calls of 12 and 500 rounds)", worst)


def test_config3_full_sampled():
    w = configs.config3()
    c = _coords(w.p, 173)
    worst, orc, gpu = harness.run_parity(w, w.rounds, every=100, coords=c, verbose=True)
    _report(w.name + f" ({c.size} sampled coordinates)", worst)


def test_config1_full():
    w = configs.config1()
    rounds = w.rounds if LONG else 1500
    # the library's defaults, automatic rebase every 512 rounds included (the rings are compared in the small case)
    worst, orc, gpu = harness.run_parity(w, rounds, every=100, verbose=True, check_rings=False)
    _report(w.name + f" ({rounds} rounds)", worst)


def test_config4_full_size():
    w = configs.config4()
    rounds = w.rounds if LONG else 200
    worst, orc, gpu = harness.run_parity(w, rounds, every=100, verbose=True, check_rings=False)
    _report(w.name + f" ({rounds} rounds)", worst)
