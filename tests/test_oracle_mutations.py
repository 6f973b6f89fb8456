"""Are the oracle's pins sharp?  Plant one plausible mistake at a time IN THE ORACLE
(a patched copy of its C source, or a patched gate), re-run a battery of the pins, and
require that at least one of them notices.  CPU only; the GPU engine is not involved.
"""
import math
import os
import subprocess

import numpy as np
import pytest

from oracle import gxpo_oracle as O
from tests import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(O.__file__), "gxpo_oracle.c")

# (name, text to find in gxpo_oracle.c, replacement)
C_MUTATIONS = [
    ("adamw: no bias correction of m", "double m_hat = m[i] / bias1;", "double m_hat = m[i];"),
    ("adamw: no bias correction of v", "double v_hat = v[i] / bias2;", "double v_hat = v[i];"),
    ("adamw: eps inside the square root", "lr * m_hat / (sqrt(v_hat) + eps)", "lr * m_hat / sqrt(v_hat + eps)"),
    ("adamw: weight decay coupled into the gradient", "double th = theta_in[i] * (1.0 - lr * weight_decay);",
     "double th = theta_in[i] - lr * weight_decay * m[i];"),
    ("adamw: weight decay dropped", "double th = theta_in[i] * (1.0 - lr * weight_decay);", "double th = theta_in[i];"),
    ("adamw: second moment uses |g| not g^2", "(1.0 - beta2) * g[i] * g[i]", "(1.0 - beta2) * fabs(g[i])"),
    ("adamw: beta1 and beta2 swapped in the moments", "m[i] = beta1 * m[i] + (1.0 - beta1) * g[i];",
     "m[i] = beta2 * m[i] + (1.0 - beta2) * g[i];"),
    ("step counter not advanced", "*step_count += 1;", "*step_count += 0;"),
    ("gd: plus instead of minus", "theta_out[i] = theta_in[i] - lr * g[i];", "theta_out[i] = theta_in[i] + lr * g[i];"),
    ("geometric sum starts at x^1", "double sum = 0.0, power = 1.0;", "double sum = 0.0, power = x;"),
    ("ratio inverted", "double r = g1 / g0;", "double r = g0 / g1;"),
    ("active set not strict", "if (!(fabs(g0) > delta32))", "if (!(fabs(g0) >= delta32))"),
    ("active set without abs", "if (!(fabs(g0) > delta32))", "if (!(g0 > delta32))"),
    ("scale = S_K / S_1", "gxpo_oracle_geometric_sum(r, K) / gxpo_oracle_geometric_sum(r, 2)",
     "gxpo_oracle_geometric_sum(r, K) / gxpo_oracle_geometric_sum(r, 1)"),
    ("scale = S_{K-1} / S_2", "gxpo_oracle_geometric_sum(r, K) / gxpo_oracle_geometric_sum(r, 2)",
     "gxpo_oracle_geometric_sum(r, K - 1) / gxpo_oracle_geometric_sum(r, 2)"),
    ("extrapolates from theta_2 instead of theta_0", "double theta_K = theta_0[i] + (theta_2[i] - theta_0[i]) * scale;",
     "double theta_K = theta_2[i] + (theta_2[i] - theta_0[i]) * scale;"),
    ("alpha blends toward theta_2 instead of theta_K", "double theta_tilde = theta_0[i] + alpha * (theta_K - theta_0[i]);",
     "double theta_tilde = theta_0[i] + alpha * (theta_2[i] - theta_0[i]);"),
    ("alpha applied as 1 - alpha", "double theta_tilde = theta_0[i] + alpha * (theta_K - theta_0[i]);",
     "double theta_tilde = theta_0[i] + (1.0 - alpha) * (theta_K - theta_0[i]);"),
    ("sum of squares sums |g|", "acc += (long double)g[i] * (long double)g[i];", "acc += fabsl((long double)g[i]);"),
    ("clamp only from above", "if (r < -R) r = -R;", ""),
    ("degenerate ratio not handled", "    if (r == -1.0)\n        return 1.0;\n    return gxpo_oracle_geometric_sum",
     "    return gxpo_oracle_geometric_sum"),
    ("bf16 truncates instead of rounding", "uint32_t rounded = b.u + 0x7fffu + kept_lsb;", "uint32_t rounded = b.u;"),
    ("bf16 rounds ties away from even", "uint32_t rounded = b.u + 0x7fffu + kept_lsb;", "uint32_t rounded = b.u + 0x8000u;"),
    ("clipping without the min", "return c < 1.0 ? c : 1.0;", "return c;"),
    ("clipping by the squared norm", "double c = max_norm / (total_norm + 1e-6);", "double c = max_norm / (total_norm * total_norm + 1e-6);"),
    ("diagnostics: cosine numerator uses g1", "a[3] += (long double)g0[i] * g_slow[i];", "a[3] += (long double)g1[i] * g_slow[i];"),
    ("diagnostics: Delta_K without the scale", "const double dK = d2 * scale;", "const double dK = d2;"),
]

BATTERY = [
    lambda: pins.test_extrapolated_point_equals_K_gd_steps(4),
    lambda: pins.test_extrapolated_point_equals_K_gd_steps(5),
    lambda: pins.test_partial_reposition_closed_form(0.5),
    lambda: pins.test_partial_reposition_closed_form(0.1),
    pins.test_scale_special_values,
    pins.test_scale_uses_g1_over_g0_not_the_inverse,
    pins.test_geometric_sum_is_the_sum,
    pins.test_active_set_is_strict_and_uses_abs,
    pins.test_inactive_and_alpha_edges_in_extrapolate,
    pins.test_degenerate_and_clamped_ratio_readings,
    lambda: pins.test_dense_quadratic_brute_force_within_paper_bound(1, 3),
    lambda: pins.test_adamw_optimstep_matches_library(0.01, 1e-8, 1e-6),
    lambda: pins.test_adamw_optimstep_matches_library(0.1, 1e-3, 1e-2),
    pins.test_gxpo_K2_alpha1_is_three_library_adamw_steps,
    pins.test_multi_tensor_equals_flat,
    pins.test_bf16_rounding_matches_library,
    lambda: pins.test_clipping_matches_library_clip_grad_norm(1.0, 5.0),
    lambda: pins.test_clipping_matches_library_clip_grad_norm(1.0, 0.05),
    pins.test_diagnostics_match_numpy_definitions,
]


def battery_fails() -> bool:
    for check in BATTERY:
        try:
            check()
        except Exception:                       # an assertion, or a NaN/inf blowing up a comparison
            return True
    return False


@pytest.fixture()
def swap_oracle_library(tmp_path):
    saved = O._lib

    def swap(source_text: str):
        c = tmp_path / "mutant.c"
        so = tmp_path / "mutant.so"
        c.write_text(source_text)
        subprocess.check_call(["gcc", "-O1", "-std=c11", "-ffp-contract=off", "-shared", "-fPIC", "-o", str(so), str(c), "-lm"])
        O._lib = None
        real_build = O.build_oracle
        O.build_oracle = lambda force=False: str(so)
        try:
            O._load()
        finally:
            O.build_oracle = real_build
    yield swap
    O._lib = saved


def test_the_unmutated_oracle_passes_the_battery():
    assert not battery_fails()


@pytest.mark.parametrize("name,old,new", C_MUTATIONS, ids=[m[0] for m in C_MUTATIONS])
def test_planted_mistake_in_the_c_oracle_is_caught(name, old, new, swap_oracle_library):
    src = open(SRC).read()
    assert src.count(old) >= 1, f"mutation anchor not found: {old!r}"
    swap_oracle_library(src.replace(old, new, 1))
    assert battery_fails(), f"no pin noticed: {name}"


# ---- the gate and the driver are Python: patch them in place -------------------------------------------
def gate_battery_fails(golden_dir) -> bool:
    checks = [lambda: pins.test_gate_statistics_match_numpy(0), lambda: pins.test_gate_statistics_match_numpy(1),
              pins.test_gate_hand_computed_threshold_is_inclusive_and_one_sided, pins.test_gate_warmup_window_and_permanence,
              lambda: pins.test_backward_pass_budget_matches_printed_table(golden_dir),
              pins.test_optimizer_state_is_not_rolled_back_on_reposition,
              lambda: pins.test_explicit_lookahead_equals_extrapolation_on_the_surrogate(3, 0.5)]
    for check in checks:
        try:
            check()
        except Exception:
            return True
    return False


def _mutant_gate_step(variant):
    def step(self, t, norm):
        c = self.cfg
        B = self.buffer
        mu = sigma = z = float("nan")
        evaluated = tripped = False
        if variant == "push first":
            B.append(norm)
        if len(B) >= c.resolved_min_count() and len(B) > c.ddof:
            evaluated = True
            mu = math.fsum(B) / len(B)
            div = len(B) - (1 - c.ddof if variant == "ddof flipped" else c.ddof)
            var = math.fsum((x - mu) ** 2 for x in B) / div
            sigma = math.sqrt(var) if variant != "variance not deviation" else var
            z = (norm - mu) / (sigma + c.eps)
            if variant == "two sided":
                z = abs(z)
            tripped = z > c.tau if variant == "strict" else z >= c.tau
        if not math.isfinite(norm):
            tripped = True
        if tripped and self.s_star is None:
            self.s_star = t if variant == "s_star = t" else t + 1
        if variant != "push first":
            B.append(norm)
        if len(B) > c.window:
            del B[0]
        if variant == "not permanent" and not tripped:
            self.s_star = None
        return O.GateInfo(norm, mu, sigma, z, evaluated, tripped, self.s_star)
    return step


@pytest.mark.parametrize("variant", ["push first", "strict", "two sided", "s_star = t", "ddof flipped",
                                     "variance not deviation", "not permanent"])
def test_planted_mistake_in_the_gate_is_caught(variant, golden_dir, monkeypatch):
    assert not gate_battery_fails(golden_dir)
    monkeypatch.setattr(O.RollingGate, "step", _mutant_gate_step(variant))
    assert gate_battery_fails(golden_dir), f"no pin noticed the gate mutation: {variant}"


def driver_battery_fails(golden_dir) -> bool:
    checks = [lambda: pins.test_extrapolated_point_equals_K_gd_steps(4), lambda: pins.test_partial_reposition_closed_form(0.5),
              pins.test_gxpo_K2_alpha1_is_three_library_adamw_steps, pins.test_parameter_groups_match_library_param_groups,
              lambda: pins.test_backward_pass_budget_matches_printed_table(golden_dir),
              pins.test_clipped_gxpo_step_is_the_unclipped_step_on_clipped_gradients,
              lambda: pins.test_explicit_lookahead_equals_extrapolation_on_the_surrogate(3, 0.5)]
    for check in checks:
        try:
            check()
        except Exception:
            return True
    return False


def _second_step_from_theta_0(self, g1):
    self.backward_passes += 1
    self._g1_used, self.norm_g1_raw, _ = O.clip_gradients(g1, self.cfg.clip_norm)
    self._theta_2 = self._optim_all(self._theta_0, self._g1_used)          # should start from theta^{t,1}
    return self._theta_2


def _slow_step_from_theta_K(self, g_slow):
    self.backward_passes += 1
    self._sumsq = [O.sum_squares(g) for g in g_slow]
    self._g_slow = [np.asarray(g, dtype=np.float64).ravel() for g in g_slow]
    used, _, _ = O.clip_gradients(g_slow, self.cfg.clip_norm)
    self.theta = self._optim_all(self.theta_K, used)                       # should start from theta~
    return self.theta


def _slow_step_not_counted(self, g_slow):
    out = _REAL["slow_step"](self, g_slow)
    self.backward_passes -= 1
    return out


def _fallback_takes_three_passes(self, g0):
    out = _REAL["fallback_step"](self, g0)
    self.backward_passes += 2
    return out


def _groups_scale_only_lr(self, thetas_in, grads):
    saved = self.weight_decay_scale
    self.weight_decay_scale = [1.0] * len(saved)
    try:
        return _REAL["_optim_all"](self, thetas_in, grads)
    finally:
        self.weight_decay_scale = saved


def _explicit_reposition_full(self):
    self.theta_tilde = [tn.copy() for tn in self._theta_j]                 # ignores alpha
    return self.theta_tilde


_REAL = {k: getattr(O.GXPOOracle, k) for k in ("slow_step", "fallback_step", "_optim_all")}
DRIVER_MUTATIONS = {
    "second fast step starts from theta^t": ("fast_step_2", _second_step_from_theta_0),
    "slow step starts from theta^{t,K}": ("slow_step", _slow_step_from_theta_K),
    "slow step's backward pass not counted": ("slow_step", _slow_step_not_counted),
    "fallback step charged three passes": ("fallback_step", _fallback_takes_three_passes),
    "parameter groups ignore the decay multiplier": ("_optim_all", _groups_scale_only_lr),
    "explicit reposition ignores alpha": ("explicit_reposition", _explicit_reposition_full),
}


@pytest.mark.parametrize("name", list(DRIVER_MUTATIONS))
def test_planted_mistake_in_the_step_driver_is_caught(name, golden_dir, monkeypatch):
    assert not driver_battery_fails(golden_dir)
    attr, mutant = DRIVER_MUTATIONS[name]
    monkeypatch.setattr(O.GXPOOracle, attr, mutant)
    assert driver_battery_fails(golden_dir), f"no pin noticed: {name}"


def test_planted_mistake_in_the_driver_is_caught(golden_dir, monkeypatch):
    # the driver restores the moments when it repositions (the paper says it must not)
    real = O.GXPOOracle.extrapolate

    def rolls_back(self, g0, g1):
        out = real(self, g0, g1)
        self.m = [np.zeros_like(x) for x in self.m] if self.m[0] is not None else self.m
        return out
    assert not gate_battery_fails(golden_dir)
    monkeypatch.setattr(O.GXPOOracle, "extrapolate", rolls_back)
    assert gate_battery_fails(golden_dir)
