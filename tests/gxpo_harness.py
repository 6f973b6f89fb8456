"""Shared plumbing of the GPU parity tests: device buffers for a tensor layout,
an oracle mirror, and the comparison rules.

Comparison rules (fp32 state against the fp64 oracle):
  * element-wise   |gpu - ref| <= rtol * |ref| + rtol * rms(ref),  rtol = 1e-5
  * displacement   ||(gpu - start) - (ref - start)||_2
                       <= dtol * ||ref - start||_2 + (2 + alpha K) * 2^-24 * ||ref||_2
    because an update of ~1e-6 on a parameter of ~2e-2 hides inside the
    element-wise bound.  dtol bounds the relative error of the update's own
    arithmetic; the second term is what storing theta in fp32 costs no matter
    how the update is computed: each stored iterate is rounded to 2^-24
    relative (theta^{t,1}, then the result), and the rounding of a stored
    theta^{t,2} is multiplied by alpha * scale <= alpha K / 2 on the way to
    theta~.
  * after the extrapolation, coordinate i may additionally differ by
    4 * 2^-24 * |theta_i| * alpha * |scale_i|: the GPU's theta^{t,1} is a stored
    fp32 number, the oracle's is not, and the extrapolation multiplies that
    storage rounding by alpha * scale_i, which is unbounded next to the pole of
    S_K/S_2 at r = -1 (odd K).
  * with gradient clipping the gradients entering the ratio are rounded products
    g * c (c itself an fp32 number), so r carries ~2^-23 relative error and the
    allowance grows by alpha * |theta^{t,2} - theta^t| * scale_i^2 * 2^-22
    (d scale / d r ~ scale^2 next to the pole).
  * bf16 model copy: bit-identical to round-to-nearest-even of the GPU's own
    fp32 result, and within 2e-2 relative of the oracle.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence

import numpy as np
import torch

from oracle import gxpo_oracle as O
from paper_2605_06755_amd import binding as B
from paper_2605_06755_amd import synth

RTOL_STATE = 1e-5
RTOL_BF16 = 2e-2


def f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a device fp32 / bf16 tensor to a host float64 array."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def assert_close(gpu: np.ndarray, ref: np.ndarray, what: str, rtol: float = RTOL_STATE, extra_abs=None):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, what
    rms = math.sqrt(float(np.mean(ref * ref))) if ref.size else 0.0
    err = np.abs(gpu - ref)
    bound = rtol * np.abs(ref) + rtol * rms
    if extra_abs is not None:
        bound = bound + extra_abs
    bad = err > bound
    if bad.any():
        i = int(np.argmax(err - bound))
        raise AssertionError(f"{what}: {int(bad.sum())}/{ref.size} outside rtol={rtol}; worst at {i}: "
                             f"gpu={gpu.flat[i]!r} ref={ref.flat[i]!r} rms={rms!r}")


def displacement_error(gpu: np.ndarray, ref: np.ndarray, start: np.ndarray) -> float:
    d_ref = ref - start
    denom = float(np.linalg.norm(d_ref))
    if denom == 0.0:
        return float(np.linalg.norm(gpu - start))
    return float(np.linalg.norm((gpu - start) - d_ref)) / denom


class DeviceState:
    """theta / theta_probe / m / v / (bf16 copy) for a list of tensor sizes, carved
    out of flat device buffers with canary padding between tensors."""

    CANARY = 12345.0

    def __init__(self, numels: Sequence[int], adam: bool, with_copy: bool, device="cuda", alternating: bool = False):
        self.numels = list(numels)
        layout = [(str(i), n) for i, n in enumerate(self.numels)]
        self.layout = layout
        total = synth.padded_numel(layout, 4) + 4
        mk = lambda dt: torch.full((total,), self.CANARY, dtype=dt, device=device)
        self.flat = {"theta": mk(torch.float32), "theta_probe": mk(torch.float32)}
        if adam:
            self.flat["m"] = mk(torch.float32)
            self.flat["v"] = mk(torch.float32)
        if alternating:                          # second buffers for the moments: the engine alternates between two sets
            self.flat["m_alt"] = mk(torch.float32)
            self.flat["v_alt"] = mk(torch.float32)
        if with_copy:
            self.flat["model_copy"] = mk(torch.bfloat16)
        self.views = {k: synth.split_like(v, layout, 4) for k, v in self.flat.items()}
        self.pad_mask = torch.ones(total, dtype=torch.bool, device=device)
        off = 0
        for n in self.numels:
            self.pad_mask[off:off + n] = False
            off += -(-n // 4) * 4
        for k in ("m", "v"):
            if k in self.views:
                for x in self.views[k]:
                    x.zero_()

    @staticmethod
    def set_keys(current_set: int):
        """Names of the parameter, first-moment and second-moment buffers of one of the two sets."""
        return ("theta_probe", "m_alt", "v_alt") if current_set else ("theta", "m", "v")

    def tensor_dicts(self) -> List[dict]:
        return [{k: self.views[k][i] for k in self.views} for i in range(len(self.numels))]

    def set_theta(self, thetas: Sequence[torch.Tensor]):
        for dst, src in zip(self.views["theta"], thetas):
            dst.copy_(src)

    def check_canaries(self):
        for k, flat in self.flat.items():
            canary = torch.tensor(self.CANARY, dtype=flat.dtype, device=flat.device)
            assert bool((flat[self.pad_mask] == canary).all()), f"padding of {k} was overwritten"

    def host(self, key: str) -> List[np.ndarray]:
        return [f64(x) for x in self.views[key]]


def grad_buffers(numels: Sequence[int], dtype, device="cuda") -> List[torch.Tensor]:
    """One gradient buffer per tensor, carved from a flat buffer (8-byte aligned for bf16)."""
    layout = [(str(i), n) for i, n in enumerate(numels)]
    flat = torch.zeros(synth.padded_numel(layout, 4) + 4, dtype=dtype, device=device)
    return synth.split_like(flat, layout, 4)


def oracle_config(cfg: B.gxpo_config) -> O.GXPOConfig:
    return O.GXPOConfig(
        optim=O.OptimConfig("adamw" if cfg.optimizer == B.GXPO_OPT_ADAMW else "gd", lr=cfg.lr, beta1=cfg.beta1,
                            beta2=cfg.beta2, eps=cfg.adam_eps, weight_decay=cfg.weight_decay),
        K=cfg.K, alpha=cfg.alpha, delta=cfg.delta, r_max=cfg.r_max, clip_norm=cfg.clip_norm,
        explicit_steps=cfg.explicit_steps,
        gate=O.GateConfig(tau=cfg.tau, window=cfg.window, eps=cfg.gate_eps, ddof=cfg.gate_ddof,
                          min_count=(cfg.gate_min_count or None)))


def sync_oracle_to_device(orc: O.GXPOOracle, dev: DeviceState, optim_steps: int, current_set: int = 0):
    """Make the oracle start a step from exactly the state the GPU holds (in the buffer set that is current)."""
    th, m, v = DeviceState.set_keys(current_set)
    orc.theta = dev.host(th)
    if "m" in dev.views:
        orc.m = dev.host(m)
        orc.v = dev.host(v)
    orc.optim_steps = optim_steps


def check_bf16_copy(dev: DeviceState, ref_thetas: Sequence[np.ndarray], what: str):
    for i, (c, th) in enumerate(zip(dev.views["model_copy"], dev.views["theta"])):
        got_bits = c.detach().cpu().view(torch.int16).numpy().view(np.uint16)
        want_bits = O.bf16_round_bits(th.detach().cpu().numpy())
        np.testing.assert_array_equal(got_bits, want_bits, err_msg=f"{what}: tensor {i} copy is not RNE(theta)")
        assert_close(O.bf16_bits_to_f64(got_bits), ref_thetas[i], f"{what}: tensor {i} bf16 copy", rtol=RTOL_BF16)


def check_bf16_copy_of(dev: DeviceState, key: str, ref_thetas: Sequence[np.ndarray], what: str):
    """model_copy must be round-to-nearest-even of the fp32 buffer `key`, and near the oracle."""
    for i, (c, th) in enumerate(zip(dev.views["model_copy"], dev.views[key])):
        got_bits = c.detach().cpu().view(torch.int16).numpy().view(np.uint16)
        np.testing.assert_array_equal(got_bits, O.bf16_round_bits(th.detach().cpu().numpy()),
                                      err_msg=f"{what}: tensor {i} copy is not RNE({key})")
        assert_close(O.bf16_bits_to_f64(got_bits), ref_thetas[i], f"{what}: tensor {i} bf16 copy", rtol=RTOL_BF16)


def lockstep_active_step(ctx: B.Context, dev: DeviceState, orc: O.GXPOOracle, grad_fn, grads, *, dtol: float,
                         fused: bool, check_copy: bool = False, what: str = ""):
    """One active step on the GPU and in the oracle from identical state and
    identical gradient buffers, compared after every call.

    grad_fn(list of device fp32 thetas, out list of grad buffers) fills the
    gradient buffers from the GPU's current parameters (the trainer's job).
    grads = (g0_bufs, g1_bufs, gs_bufs); g_slow may share g0's buffers.
    Returns (gate info from GPU, gate info from oracle).
    """
    g0b, g1b, gsb = grads
    st = B.gxpo_get_state(ctx)
    # where things are: in place, theta / m / v hold the state throughout and theta_probe the first probe; with
    # alternating state (the tensors brought m_alt, v_alt) the state moves between the two sets as the header says
    alternating = "m_alt" in dev.views
    c0 = st.current_set
    assert alternating or c0 == 0
    K_TH, K_M, K_V = DeviceState.set_keys(c0)                       # the set that holds theta^t
    K_PROBE = DeviceState.set_keys(1 - c0)[0] if alternating else "theta_probe"
    K_TH2, K_M2, K_V2 = DeviceState.set_keys(1 - c0) if alternating else (K_TH, K_M, K_V)       # where theta~ goes
    sync_oracle_to_device(orc, dev, st.optim_steps, c0)
    start = dev.host(K_TH)
    adam = "m" in dev.views
    m_start, v_start = (dev.host(K_M), dev.host(K_V)) if adam else (None, None)

    def compare(key_gpu: str, ref_list, label, disp_from=None, amplified=False):
        got = dev.host(key_gpu)
        for i, (g, r) in enumerate(zip(got, ref_list)):
            extra = None
            if amplified:
                extra = 4.0 * 2.0 ** -24 * np.abs(r) * ctx.cfg.alpha * np.abs(orc.scale[i])
                if ctx.cfg.clip_norm > 0:
                    # clipped gradients are rounded products and the factor itself is an fp32 number:
                    # the ratio carries ~2^-23 relative error, and d scale / d r ~ scale^2 next to the pole
                    extra = extra + ctx.cfg.alpha * np.abs(orc._theta_2[i] - orc._theta_0[i]) * orc.scale[i] ** 2 * 2.0 ** -22
            assert_close(g, r, f"{what} {label} tensor {i}", extra_abs=extra)
        if disp_from is not None:
            num = math.sqrt(sum(float(np.sum(((g - s) - (r - s)) ** 2)) for g, r, s in zip(got, ref_list, disp_from)))
            den = math.sqrt(sum(float(np.sum((r - s) ** 2)) for r, s in zip(ref_list, disp_from)))
            ref_norm = math.sqrt(sum(float(np.sum(r * r)) for r in ref_list))
            floor = (2.0 + ctx.cfg.alpha * ctx.cfg.K) * 2.0 ** -24 * ref_norm
            assert num <= dtol * den + floor, (f"{what} {label}: displacement error {num:.3e} vs displacement {den:.3e} "
                                               f"(dtol {dtol}, fp32 storage floor {floor:.3e})")

    def compare_moments(label, km=K_M, kv=K_V):
        if adam:
            compare(km, orc.m, label + " m")
            compare(kv, orc.v, label + " v")

    # fast step 1
    grad_fn(dev.views[K_TH], g0b)
    B.gxpo_fast_steps(ctx, 0, g0b)
    ref1 = orc.fast_step_1([f64(g) for g in g0b])
    compare(K_PROBE, ref1, "theta^{t,1}", start)
    if fused:
        # the probe pass only previews the step: the stored moments are advanced by gxpo_extrapolate
        if adam:
            for k, before in ((K_M, m_start), (K_V, v_start)):
                for g, b in zip(dev.host(k), before):
                    np.testing.assert_array_equal(g, b, err_msg=f"{what}: {k} changed by the probe pass of the fused schedule")
    else:
        compare_moments("after fast step 1")
    for g, s in zip(dev.host(K_TH), start):
        np.testing.assert_array_equal(g, s, err_msg=f"{what}: theta^t modified by the first fast step")
    # fast step 2
    grad_fn(dev.views[K_PROBE], g1b)
    B.gxpo_fast_steps(ctx, 1, g1b)
    ref2 = orc.fast_step_2([f64(g) for g in g1b])
    if not fused:
        compare("theta_probe", ref2, "theta^{t,2}", start)
        compare_moments("after fast step 2")
    # extrapolate + reposition
    B.gxpo_extrapolate(ctx, g0b, g1b)
    assert B.gxpo_get_state(ctx).current_set == (1 - c0 if alternating else 0)
    ref_t = orc.extrapolate([f64(g) for g in g0b], [f64(g) for g in g1b])
    compare(K_TH2, ref_t, "theta~", start, amplified=True)
    compare_moments("after extrapolate", K_M2, K_V2)
    if alternating:                                                 # the set that was read still holds the step's start
        for k, before in ((K_TH, start), (K_M, m_start), (K_V, v_start)):
            for g, b in zip(dev.host(k), before):
                np.testing.assert_array_equal(g, b, err_msg=f"{what}: {k} (the set gxpo_extrapolate reads) changed")
    if check_copy and (ctx.cfg.copy_mask & B.GXPO_COPY_AT_TILDE):
        check_bf16_copy_of(dev, K_TH2, ref_t, what + " theta~")
    # slow step
    grad_fn(dev.views[K_TH2], gsb)
    gs_host = [f64(g) for g in gsb]
    B.gxpo_slow_step(ctx, gsb)
    assert B.gxpo_get_state(ctx).current_set == c0
    ref_n = orc.slow_step(gs_host)
    compare(K_TH, ref_n, "theta^{t+1}", start, amplified=True)
    compare_moments("after slow step")
    if check_copy and (ctx.cfg.copy_mask & B.GXPO_COPY_AT_FINAL):
        check_bf16_copy_of(dev, K_TH, ref_n, what + " theta^{t+1}")
    # gate
    info = B.gxpo_gate(ctx)
    ref_info = orc.gate_step()
    assert info.norm == pytest_approx(ref_info.norm, 1e-12), f"{what}: norm {info.norm!r} vs {ref_info.norm!r}"
    got_tn = B.gxpo_tensor_norms(ctx)
    for a, b in zip(got_tn, orc.tensor_norms()):
        assert a == pytest_approx(b, 1e-12), f"{what}: tensor norm {a!r} vs {b!r}"
    assert bool(info.evaluated) == ref_info.evaluated
    if ref_info.evaluated:
        assert info.mu == pytest_approx(ref_info.mu, 1e-12)
        assert abs(info.z - ref_info.z) <= 1e-6 * max(1.0, abs(ref_info.z)), f"{what}: Z {info.z!r} vs {ref_info.z!r}"
    assert bool(info.tripped) == ref_info.tripped
    assert (info.s_star if info.s_star >= 0 else None) == ref_info.s_star
    if ctx.cfg.diagnostics:
        check_diagnostics(B.gxpo_get_diagnostics(ctx), orc.diagnostics(), aliased=any(a.data_ptr() == b.data_ptr() for a, b in zip(g0b, gsb)),
                          what=what)
    dev.check_canaries()
    return info, ref_info


def check_diagnostics(got, ref: dict, aliased: bool, what: str = ""):
    """Engine diagnostics against the oracle's.  The sums are fp64 on both sides; what differs
    is that the engine forms r, scale and the displacements in fp32."""
    def close(name, rel, abs_=0.0):
        a, b = getattr(got, name), ref[name]
        assert abs(a - b) <= rel * abs(b) + abs_, f"{what}: {name} {a!r} vs oracle {b!r}"
    close("norm_g0", 1e-12); close("norm_g1", 1e-12); close("norm_g_slow", 1e-12)
    if aliased:
        assert math.isnan(got.cos_g0_g_slow), f"{what}: cosine must be NaN when g_slow overwrote g0"
    else:
        close("cos_g0_g_slow", 1e-10, 1e-12)
    close("inactive_fraction", 1e-12, 1e-15)
    close("retention_mean", 1e-6)
    close("retention_std", 1e-4, 1e-9)
    close("scale_mean", 1e-5)
    close("displacement_ratio", 1e-4)


class pytest_approx:
    """Relative comparison usable inside plain asserts (keeps this module free of pytest)."""

    def __init__(self, ref: float, rel: float):
        self.ref, self.rel = ref, rel

    def __eq__(self, other):
        return abs(other - self.ref) <= self.rel * abs(self.ref)

    __req__ = __eq__
