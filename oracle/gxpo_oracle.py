"""fp64 CPU oracle for the GXPO parameter-space update -- TEST INFRASTRUCTURE.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this module.  It shares nothing with the HIP engine:
the element-wise arithmetic lives in ``gxpo_oracle.c`` (plain C, fp64), and
this file adds the step-by-step driver of Algorithm 1 and the rolling
z-score gate, both in plain Python on top of those C routines.

Everything follows Algorithm 1 of the paper in the paper's order:

    theta^{t,1} = OptimStep(theta^t,     g^{t,0})
    theta^{t,2} = OptimStep(theta^{t,1}, g^{t,1})
    scale       = S_K(r)/S_2(r) on the active set, 1 elsewhere
    theta^{t,K} = theta^t + (theta^{t,2} - theta^t) * scale
    theta~^t    = theta^t + alpha (theta^{t,K} - theta^t)
    theta^{t+1} = OptimStep(theta~^t, g_slow^t)
    gate on ||g_slow^t||_2, then push it into the rolling buffer

and, once the gate has tripped, theta^{t+1} = OptimStep(theta^t, g^{t,0}).

Parity status of the pieces (see tests/test_oracle_pins.py):
  * OptimStep (GD, AdamW), extrapolation, reposition, norm, step counting and
    the backward-pass budget are pinned to closed forms, brute-force unrolls,
    a library AdamW and the paper's printed table.
  * parity unpinned: the gate constants the paper never states (window w,
    epsilon, population-vs-sample deviation, warm-up length), the r = -1 and
    r_max readings, and the non-finite-norm rule.  They follow the readings
    documented next to each function and are exercised only by hand-computed
    examples.
  * parity unpinned against the paper, pinned against something else: the
    mechanism diagnostics (the paper names the quantities, not their formulas;
    pinned to numpy definitions and closed forms on the diagonal surrogate),
    global-norm clipping (the paper gives only the threshold; pinned to the
    library routine), the explicit n-step lookahead (the paper only names the
    scheme; pinned to brute-force gradient descent and to the extrapolation on
    the diagonal surrogate) and parameter groups (not in the paper; pinned to a
    library AdamW with parameter groups).
How sharp the pins are is tested by planting mistakes (tests/test_oracle_mutations.py).
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass, field, replace
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gxpo_oracle.c")
_LIB = os.path.join(_HERE, "libgxpo_oracle.so")


def build_oracle(force: bool = False) -> str:
    """Compile gxpo_oracle.c with gcc (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-Wall", "-Wextra",
             "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None
_dp = ctypes.POINTER(ctypes.c_double)


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build_oracle())
    lib.gxpo_oracle_optim_step.restype = None
    lib.gxpo_oracle_optim_step.argtypes = [
        ctypes.c_int, ctypes.c_double, ctypes.c_double, ctypes.c_double,
        ctypes.c_double, ctypes.c_double, ctypes.c_int64,
        ctypes.POINTER(ctypes.c_int64), _dp, _dp, _dp, _dp, _dp]
    lib.gxpo_oracle_geometric_sum.restype = ctypes.c_double
    lib.gxpo_oracle_geometric_sum.argtypes = [ctypes.c_double, ctypes.c_int]
    lib.gxpo_oracle_scale.restype = ctypes.c_double
    lib.gxpo_oracle_scale.argtypes = [ctypes.c_double, ctypes.c_double, ctypes.c_int,
                                      ctypes.c_double, ctypes.c_double]
    lib.gxpo_oracle_extrapolate.restype = None
    lib.gxpo_oracle_extrapolate.argtypes = [
        ctypes.c_int64, _dp, _dp, _dp, _dp, ctypes.c_int, ctypes.c_double,
        ctypes.c_double, ctypes.c_double, _dp, _dp, _dp]
    lib.gxpo_oracle_sum_squares.restype = ctypes.c_double
    lib.gxpo_oracle_sum_squares.argtypes = [ctypes.c_int64, _dp]
    lib.gxpo_oracle_clip_coefficient.restype = ctypes.c_double
    lib.gxpo_oracle_clip_coefficient.argtypes = [ctypes.c_double, ctypes.c_double]
    lib.gxpo_oracle_diagnostic_sums.restype = None
    lib.gxpo_oracle_diagnostic_sums.argtypes = [
        ctypes.c_int64, _dp, _dp, _dp, _dp, _dp, ctypes.c_int, ctypes.c_double, ctypes.c_double, ctypes.c_double, _dp]
    lib.gxpo_oracle_bf16_bits.restype = ctypes.c_uint16
    lib.gxpo_oracle_bf16_bits.argtypes = [ctypes.c_float]
    lib.gxpo_oracle_bf16_round_array.restype = None
    lib.gxpo_oracle_bf16_round_array.argtypes = [
        ctypes.c_int64, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_uint16)]
    _lib = lib
    return lib


def _f64(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a


def _p(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.cast(None, _dp)
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_dp)


# ---------------------------------------------------------------------------
# thin array-level wrappers around the C routines
# ---------------------------------------------------------------------------
@dataclass
class OptimConfig:
    """OptimStep hyper-parameters.  optimizer: 'gd' or 'adamw'."""
    optimizer: str = "adamw"
    lr: float = 1e-6
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01


def optim_step(cfg: OptimConfig, step_count: int, theta: np.ndarray, g: np.ndarray,
               m: Optional[np.ndarray], v: Optional[np.ndarray]):
    """One OptimStep.  Returns (theta_new, new_step_count); m, v updated in place."""
    lib = _load()
    theta = _f64(theta)
    g = _f64(g)
    out = np.empty_like(theta)
    cnt = ctypes.c_int64(step_count)
    opt = {"gd": 0, "adamw": 1}[cfg.optimizer]
    if opt == 1:
        assert m is not None and v is not None
    lib.gxpo_oracle_optim_step(opt, cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay,
                               theta.size, ctypes.byref(cnt), _p(theta.ravel()), _p(g.ravel()),
                               _p(m), _p(v), _p(out.ravel()))
    return out, cnt.value


def geometric_sum(x: float, n: int) -> float:
    return _load().gxpo_oracle_geometric_sum(float(x), int(n))


def scale_factor(g0: float, g1: float, K: int, delta: float, r_max: float = math.inf) -> float:
    return _load().gxpo_oracle_scale(float(g0), float(g1), int(K), float(delta), float(r_max))


def extrapolate(theta_0, theta_2, g0, g1, K: int, alpha: float, delta: float,
                r_max: float = math.inf):
    """Returns (scale, theta_K, theta_tilde) as float64 arrays."""
    lib = _load()
    theta_0, theta_2, g0, g1 = (_f64(a).ravel() for a in (theta_0, theta_2, g0, g1))
    n = theta_0.size
    assert theta_2.size == n and g0.size == n and g1.size == n
    scale = np.empty(n)
    theta_K = np.empty(n)
    theta_t = np.empty(n)
    lib.gxpo_oracle_extrapolate(n, _p(theta_0), _p(theta_2), _p(g0), _p(g1), int(K),
                                float(alpha), float(delta), float(r_max),
                                _p(scale), _p(theta_K), _p(theta_t))
    return scale, theta_K, theta_t


def sum_squares(g) -> float:
    g = _f64(g).ravel()
    return _load().gxpo_oracle_sum_squares(g.size, _p(g))


def clip_coefficient(total_norm: float, max_norm: float) -> float:
    return _load().gxpo_oracle_clip_coefficient(float(total_norm), float(max_norm))


def clip_gradients(grads, max_norm: float):
    """Global-norm clipping of one gradient (a list of tensors): returns
    (clipped list, total norm before clipping, coefficient)."""
    arrs = [_f64(g).ravel() for g in grads]
    total = math.sqrt(math.fsum(sum_squares(a) for a in arrs))
    c = _load().gxpo_oracle_clip_coefficient(total, float(max_norm))
    return [a * c for a in arrs], total, c


def diagnostics(theta_0s, theta_2s, g0s, g1s, g_slows, K: int, delta: float, r_max: float = math.inf) -> dict:
    """Mechanism diagnostics of one active step over a list of tensors (the
    quantities of the paper's appendix table of active-phase diagnostics)."""
    lib = _load()
    arrs = [[_f64(a).ravel() for a in lst] for lst in (theta_0s, theta_2s, g0s, g1s, g_slows)]

    def sums(mean_r):
        tot = np.zeros(10)
        for th0, th2, a, b, c in zip(*arrs):
            out = np.zeros(10)
            lib.gxpo_oracle_diagnostic_sums(th0.size, _p(th0), _p(th2), _p(a), _p(b), _p(c), int(K), float(delta),
                                            float(r_max), float(mean_r), _p(out))
            tot += out
        return tot
    first = sums(float("nan"))
    n_total = sum(a.size for a in arrs[0])
    n_act = first[4]
    mean_r = first[5] / n_act if n_act else float("nan")
    s = sums(mean_r) if n_act else first
    ng0, ng1, ngs = math.sqrt(s[0]), math.sqrt(s[1]), math.sqrt(s[2])
    return {
        "norm_g0": ng0, "norm_g1": ng1, "norm_g_slow": ngs,
        "cos_g0_g_slow": s[3] / (ng0 * ngs) if ng0 > 0 and ngs > 0 else float("nan"),
        "retention_mean": mean_r,
        "retention_std": math.sqrt(s[6] / n_act) if n_act else float("nan"),
        "scale_mean": s[7] / n_act if n_act else float("nan"),
        "inactive_fraction": 1.0 - n_act / n_total,
        "displacement_ratio": math.sqrt(s[9] / s[8]) if s[8] > 0 else float("nan"),
    }


def bf16_round_bits(x32: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 array of bf16 bit patterns (round-to-nearest-even)."""
    x32 = np.ascontiguousarray(x32, dtype=np.float32).ravel()
    out = np.empty(x32.size, dtype=np.uint16)
    _load().gxpo_oracle_bf16_round_array(
        x32.size, x32.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
        out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)))
    return out


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of stored bf16 bit patterns (input marshalling only)."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return u.view(np.float32).astype(np.float64)


# ---------------------------------------------------------------------------
# rolling z-score gate (Section 2.3 "Adaptive rule in practice", Eq. (10);
# Algorithm 1, the block after the slow correction)
# ---------------------------------------------------------------------------
@dataclass
class GateConfig:
    """Gate constants.

    tau        trigger threshold (paper: tau).
    window     w, how many past norms the statistics look at.  READING: the
               paper never gives w.
    eps        epsilon of Eq. (10).  READING: never given; 1e-8 here.
    ddof       0 = population deviation, 1 = sample deviation.  READING: the
               paper says only "standard deviation"; population is the default.
    min_count  the gate is evaluated only when the buffer already holds at
               least this many norms.  READING: the text says warm-up only
               fills the buffer and that the statistics are over the past w
               norms, the algorithm listing tests len(B) > 1; `window` (the
               text) is the default, 2 (the listing) is selectable.
    """
    tau: float = 3.0
    window: int = 10
    eps: float = 1e-8
    ddof: int = 0
    min_count: Optional[int] = None

    def resolved_min_count(self) -> int:
        return self.window if self.min_count is None else self.min_count


@dataclass
class GateInfo:
    norm: float
    mu: float
    sigma: float
    z: float
    evaluated: bool
    tripped: bool
    s_star: Optional[int]


class RollingGate:
    """Rolling buffer B of recent ||g_slow||_2 and the trip rule Z_t >= tau."""

    def __init__(self, cfg: GateConfig):
        self.cfg = cfg
        self.buffer: List[float] = []
        self.s_star: Optional[int] = None      # None stands for +infinity

    def step(self, t: int, norm: float) -> GateInfo:
        """Evaluate the gate for training step t, THEN insert the norm.

        The statistics are those of the buffer before the current norm goes
        in (Section 2.3, sentence introducing Eq. (10)).  Z_t >= tau sets
        s* = t + 1 for good.  READING: a non-finite norm trips the gate (a NaN
        comparison would otherwise never fire).  The tripping norm is still
        pushed (Algorithm 1 updates the buffer unconditionally).
        """
        c = self.cfg
        B = self.buffer
        mu = sigma = z = float("nan")
        evaluated = False
        tripped = False
        if len(B) >= c.resolved_min_count() and len(B) > c.ddof:
            evaluated = True
            mu = math.fsum(B) / len(B)
            var = math.fsum((x - mu) ** 2 for x in B) / (len(B) - c.ddof)
            sigma = math.sqrt(var)
            z = (norm - mu) / (sigma + c.eps)
            tripped = z >= c.tau
        if not math.isfinite(norm):
            tripped = True
        if tripped and self.s_star is None:
            self.s_star = t + 1
        B.append(norm)
        if len(B) > c.window:
            del B[0]
        return GateInfo(norm, mu, sigma, z, evaluated, tripped, self.s_star)


# ---------------------------------------------------------------------------
# Algorithm 1, step by step, over a list of parameter tensors
# ---------------------------------------------------------------------------
@dataclass
class GXPOConfig:
    optim: OptimConfig = field(default_factory=OptimConfig)
    K: int = 8
    alpha: float = 0.5
    delta: float = 1e-8
    r_max: float = math.inf
    clip_norm: float = 0.0          # 0 = no clipping
    explicit_steps: int = 0         # n >= 2: take n real fast steps instead of extrapolating (see explicit_*)
    gate: GateConfig = field(default_factory=GateConfig)


class GXPOOracle:
    """Holds theta, AdamW moments, the optimizer step counter, B and s*.

    The caller plays the trainer: it evaluates gradients wherever the
    algorithm asks for them and hands them in.  `backward_passes` counts the
    gradient hand-offs, which is the paper's cost unit (3 per active step,
    1 per fallback step).
    """

    def __init__(self, cfg: GXPOConfig, thetas: Sequence[np.ndarray]):
        self.cfg = cfg
        self.theta = [_f64(np.array(t, dtype=np.float64)).ravel().copy() for t in thetas]
        adam = cfg.optim.optimizer == "adamw"
        self.m = [np.zeros_like(t) if adam else None for t in self.theta]
        self.v = [np.zeros_like(t) if adam else None for t in self.theta]
        self.optim_steps = 0
        self.t = 0
        self.gate = RollingGate(cfg.gate)
        self.backward_passes = 0
        # per-step scratch
        self._theta_0 = None
        self._theta_1 = None
        self._theta_2 = None
        self.theta_K = None
        self.theta_tilde = None
        self.scale = None
        self._sumsq = None
        self._g0 = self._g1 = self._g_slow = None
        # parameter groups: per-tensor multipliers of lr and weight_decay (all 1 = the paper's uniform setting)
        self.lr_scale = [1.0] * len(self.theta)
        self.weight_decay_scale = [1.0] * len(self.theta)

    # -- phase ----------------------------------------------------------------
    @property
    def s_star(self):
        return self.gate.s_star

    def is_active(self) -> bool:
        return self.gate.s_star is None or self.t < self.gate.s_star

    def _optim_all(self, thetas_in, grads):
        """OptimStep on every tensor with one shared step counter."""
        outs = []
        new_count = self.optim_steps
        for i, (th, g, m, v) in enumerate(zip(thetas_in, grads, self.m, self.v)):
            oc = self.cfg.optim
            if self.lr_scale[i] != 1.0 or self.weight_decay_scale[i] != 1.0:
                # READING (the paper trains with one uniform setting): a parameter group is the same
                # OptimStep with its own learning rate and weight decay, as optimizer libraries define it
                oc = replace(oc, lr=oc.lr * self.lr_scale[i], weight_decay=oc.weight_decay * self.weight_decay_scale[i])
            out, new_count = optim_step(oc, self.optim_steps, th, _f64(g).ravel(), m, v)
            outs.append(out)
        self.optim_steps = new_count
        return outs

    # -- active phase -----------------------------------------------------------
    def fast_step_1(self, g0):
        """theta^{t,1} = OptimStep(theta^t, g^{t,0}); theta^t is kept."""
        assert self.is_active()
        self.backward_passes += 1
        self._theta_0 = [t.copy() for t in self.theta]
        self._g0_used, self.norm_g0_raw, _ = clip_gradients(g0, self.cfg.clip_norm)
        self._theta_1 = self._optim_all(self._theta_0, self._g0_used)
        return self._theta_1

    def fast_step_2(self, g1):
        """theta^{t,2} = OptimStep(theta^{t,1}, g^{t,1})."""
        self.backward_passes += 1
        self._g1_used, self.norm_g1_raw, _ = clip_gradients(g1, self.cfg.clip_norm)
        self._theta_2 = self._optim_all(self._theta_1, self._g1_used)
        return self._theta_2

    def extrapolate(self, g0, g1):
        """Active set, ratio, scale, theta^{t,K}, theta~^t.  READING: with clipping the ratio
        is formed from the gradients the two fast steps consumed, i.e. after clipping."""
        c = self.cfg
        self._g0 = [_f64(g).ravel() for g in g0]
        self._g1 = [_f64(g).ravel() for g in g1]
        if c.clip_norm > 0:
            g0, g1 = self._g0_used, self._g1_used
        self.scale, self.theta_K, self.theta_tilde = [], [], []
        for th0, th2, a, b in zip(self._theta_0, self._theta_2, g0, g1):
            s, tk, tt = extrapolate(th0, th2, a, b, c.K, c.alpha, c.delta, c.r_max)
            self.scale.append(s)
            self.theta_K.append(tk)
            self.theta_tilde.append(tt)
        return self.theta_tilde

    # -- explicit lookahead: the slow-fast scheme GXPO is compared with ---------------------
    # Section 1 describes it as K fast inner steps followed by a slow correction, K + 1
    # backward passes per update.  Here: n real OptimSteps from theta^t, the same partial
    # reposition theta~ = theta^t + alpha (theta^{t,n} - theta^t) with no extrapolation
    # factor, then the usual slow step and gate.
    def explicit_fast_step(self, j: int, g):
        """theta^{t,j+1} = OptimStep(theta^{t,j}, g), j = 0 .. n-1 (theta^{t,0} = theta^t)."""
        assert self.is_active() and 0 <= j < self.cfg.explicit_steps
        self.backward_passes += 1
        used, _, _ = clip_gradients(g, self.cfg.clip_norm)
        if j == 0:
            self._theta_0 = [t.copy() for t in self.theta]
            self._theta_j = self._theta_0
        self._theta_j = self._optim_all(self._theta_j, used)
        return self._theta_j

    def explicit_reposition(self):
        """theta~ = theta^t + alpha (theta^{t,n} - theta^t)."""
        a = self.cfg.alpha
        self.theta_tilde = [t0 + a * (tn - t0) for t0, tn in zip(self._theta_0, self._theta_j)]
        return self.theta_tilde

    def slow_step(self, g_slow):
        """theta^{t+1} = OptimStep(theta~^t, g_slow); records sum g_slow^2 per tensor."""
        self.backward_passes += 1
        self._sumsq = [sum_squares(g) for g in g_slow]        # the gate sees the norm before clipping
        self._g_slow = [_f64(g).ravel() for g in g_slow]
        used, _, _ = clip_gradients(g_slow, self.cfg.clip_norm)
        self.theta = self._optim_all(self.theta_tilde, used)
        return self.theta

    def diagnostics(self) -> dict:
        """Mechanism diagnostics of the step whose slow correction just ran."""
        c = self.cfg
        if c.clip_norm > 0:
            # ratio statistics follow the gradients the fast steps consumed; norms are those handed in
            d = diagnostics(self._theta_0, self._theta_2, self._g0_used, self._g1_used, self._g_slow, c.K, c.delta, c.r_max)
            d["norm_g0"], d["norm_g1"] = self.norm_g0_raw, self.norm_g1_raw
            return d
        return diagnostics(self._theta_0, self._theta_2, self._g0, self._g1, self._g_slow, c.K, c.delta, c.r_max)

    def tensor_norms(self):
        return [math.sqrt(s) for s in self._sumsq]

    def gate_step(self) -> GateInfo:
        """Z-score test on ||g_slow||_2 over all tensors, then t <- t + 1."""
        norm = math.sqrt(math.fsum(self._sumsq))
        info = self.gate.step(self.t, norm)
        self.t += 1
        return info

    # -- fallback phase ---------------------------------------------------------
    def fallback_step(self, g0):
        """theta^{t+1} = OptimStep(theta^t, g^{t,0}); single-pass GRPO update."""
        assert not self.is_active()
        self.backward_passes += 1
        used, _, _ = clip_gradients(g0, self.cfg.clip_norm)
        self.theta = self._optim_all(self.theta, used)
        self.t += 1
        return self.theta

    # -- convenience: a whole training step with a gradient callback -------------
    def train_step(self, grad_fn):
        """grad_fn(list_of_theta_arrays) -> list of gradient arrays."""
        if self.is_active():
            g0 = grad_fn(self.theta)
            th1 = self.fast_step_1(g0)
            g1 = grad_fn(th1)
            self.fast_step_2(g1)
            tt = self.extrapolate(g0, g1)
            gs = grad_fn(tt)
            self.slow_step(gs)
            return self.gate_step()
        g0 = grad_fn(self.theta)
        self.fallback_step(g0)
        return None
