"""The pins must notice plausible mistakes: each mutant below is the oracle's own
source with one planted error (a dropped term, a wrong sign or index, a skipped
rule); at least one pin has to fail on it.  Everything runs on the CPU."""
import importlib.util
import os
import sys
import types

import numpy as np
import pytest

import test_oracle_pins as pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = open(os.path.join(ROOT, "oracle", "rfast_oracle.py")).read()

MUTANTS = {
    "descent_sign": ("v_new = self.x[i] - gamma * self.z[i]", "v_new = self.x[i] + gamma * self.z[i]"),
    "self_weight_dropped": ("x_new = self.r_self[i] * v_new", "x_new = 1.0 * v_new"),
    "mix_reads_own_slot": ("x_new = x_new + w * self.v[j][int(stamp_v[e])]", "x_new = x_new + w * self.v[j][int(self.t[j])]"),
    "buffer_not_subtracted": ("z_half = z_half + (consumed[e] - self.rho_tilde[e])", "z_half = z_half + consumed[e]"),
    "old_gradient_kept_in": ("z_half = z_half + g_new - self.g[i]", "z_half = z_half + g_new"),
    "keep_unscaled": ("z_new = self.c_self[i] * z_half", "z_new = z_half"),
    "push_with_self_weight": ("self.rho[e][t + 1] = self.rho[e][t] + w * z_half", "self.rho[e][t + 1] = self.rho[e][t] + self.c_self[i] * z_half"),
    "push_not_cumulative": ("self.rho[e][t + 1] = self.rho[e][t] + w * z_half", "self.rho[e][t + 1] = w * z_half"),
    "publishes_x_instead_of_v": ("self.v[i][t + 1] = v_new", "self.v[i][t + 1] = x_new"),
    "buffer_not_updated": ("self.rho_tilde[e] = consumed[e].copy()", "pass"),
    "delay_ignored": ("u = int(self.t_start[max(r - int(delay_C[e]), 0)][j])", "u = int(self.t_start[r][j])"),
    "delay_off_by_one": ("u = int(self.t_start[max(r - int(delay_R[e]), 0)][j])", "u = int(self.t_start[max(r - int(delay_R[e]) - 1, 0)][j])"),
    "loss_ignored": ("return all(not hist.get(t - k, True) for k in range(1, self.burst))", "return True"),
    "stamps_not_monotone": ("sr[e] = max(int(self.tau_rho[e]), cand)", "sr[e] = cand"),
    "forced_delivery_missing": ("return all(not hist.get(t - k, True) for k in range(1, self.burst))", "return False"),
    "gradient_sample_stamp": ("g_new = self._sample(i, x_new, t + 1, batch)", "g_new = self._sample(i, x_new, t, batch)"),
}

PINS = [
    pins.test_hand_stepped_n3_example_exact,
    lambda: pins.test_tracking_conservation_and_running_sum(0),
    pins.test_resolver_properties_and_mailbox_bruteforce,
    pins.test_synchronous_reduction_matches_dense_recursion,
    lambda: pins.test_dense_augmented_system_cross_formulation(0),
    pins.test_serialisation_equivalence,
    pins.test_sample_stamp_convention,
    lambda: pins.test_fixed_point_diag_quadratic_closed_form("biring"),
]


def _mutant_class(old, new):
    assert SRC.count(old) == 1, old
    mod = types.ModuleType("oracle_mutant")
    exec(compile(SRC.replace(old, new), "oracle_mutant", "exec"), mod.__dict__)
    return mod.RFastOracle


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_planted_mistake(name, monkeypatch):
    old, new = MUTANTS[name]
    monkeypatch.setattr(pins, "RFastOracle", _mutant_class(old, new))
    caught = []
    for pin in PINS:
        try:
            pin()
        except (AssertionError, KeyError, ValueError, StopIteration, RuntimeError) as exc:
            caught.append(type(exc).__name__)
            break
    assert caught, f"no pin noticed the planted mistake '{name}'"


def test_unmutated_source_passes_the_same_pins(monkeypatch):
    mod = types.ModuleType("oracle_copy")
    exec(compile(SRC, "oracle_copy", "exec"), mod.__dict__)
    monkeypatch.setattr(pins, "RFastOracle", mod.RFastOracle)
    for pin in PINS[:5]:
        pin()


# ------------------------------------------------ the labelled optimizer variant
import test_oracle_optimizer as opt_pins

OPT_MUTANTS = {
    "buffer_takes_gradient": ("self.m[i] = self.momentum * self.m[i] + self.z[i]", "self.m[i] = self.momentum * self.m[i] + self.g[i]"),
    "buffer_not_damped": ("self.m[i] = self.momentum * self.m[i] + self.z[i]", "self.m[i] = self.m[i] + self.z[i]"),
    "descent_ignores_buffer": ("v_new = self.x[i] - gamma * self.m[i]", "v_new = self.x[i] - gamma * self.z[i]"),
    "decay_missing_at_init": ("self._sample(i, self.x[i], 0, None if batch0 is None else batch0[i])",
                              "self.obj.grad(i, self.x[i], 0, None if batch0 is None else batch0[i])"),
    "decay_at_old_point": ("g_new = self._sample(i, x_new, t + 1, batch)",
                           "g_new = self.obj.grad(i, x_new, t + 1, batch) + self.weight_decay * self.x[i]"),
    "decay_sign": ("return g + self.weight_decay * x if", "return g - self.weight_decay * x if"),
}

OPT_PINS = [
    lambda: opt_pins.test_one_node_is_textbook_sgd(0.9, 1e-2),
    opt_pins.test_momentum_first_steps_by_hand,
    opt_pins.test_tracking_identity_and_untouched_buffers,
]


@pytest.mark.parametrize("name", sorted(OPT_MUTANTS))
def test_optimizer_pins_catch_planted_mistake(name, monkeypatch):
    old, new = OPT_MUTANTS[name]
    monkeypatch.setattr(opt_pins, "RFastOracle", _mutant_class(old, new))
    caught = False
    for pin in OPT_PINS:
        try:
            pin()
        except AssertionError:
            caught = True
            break
    assert caught, f"no pin noticed the planted mistake '{name}'"
