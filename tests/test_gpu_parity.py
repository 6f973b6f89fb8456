"""GPU parity: the HIP engine, called through the C ABI, against the fp64 oracle.

Sizes here are ones the oracle finishes in seconds but that still span many
blocks (a block covers 256 elements by default) and ragged tails; the
full-size workloads are in test_gpu_fullsize.py.
"""
import math

import numpy as np
import pytest
import torch

from oracle import gxpo_oracle as O
from paper_2605_06755_amd import binding as B
from paper_2605_06755_amd import synth
from tests import gxpo_harness as H

pytestmark = pytest.mark.gpu

RAGGED = [1, 2, 3, 5, 255, 256, 257, 1000, 1024, 4099, 65536 + 5, 3 * 256 * 64 + 7, 100003]


def quad_trainer(problem, numels, sigma=None, step_noise=None):
    """Returns grad_fn(list of theta views, out buffers) for a flat problem split by numels."""
    offs = np.concatenate([[0], np.cumsum(numels)])

    def grad_fn(thetas, outs):
        flat = torch.cat([t.reshape(-1) for t in thetas])
        g = synth.quadratic_grad(problem, flat, step_noise() if step_noise else None, sigma, out_dtype=outs[0].dtype)
        for i, o in enumerate(outs):
            o.copy_(g[offs[i]:offs[i + 1]])
    return grad_fn


def build(numels, cfg, problem, with_copy=False, alternating=False):
    adam = cfg.optimizer == B.GXPO_OPT_ADAMW
    dev = H.DeviceState(numels, adam, with_copy, alternating=alternating)
    offs = np.concatenate([[0], np.cumsum(numels)])
    dev.set_theta([problem.theta_0[offs[i]:offs[i + 1]] for i in range(len(numels))])
    ctx = B.gxpo_init(cfg, dev.tensor_dicts())
    orc = O.GXPOOracle(H.oracle_config(cfg), dev.host("theta"))
    gdt = torch.float32 if cfg.grad_dtype == B.GXPO_GRAD_F32 else torch.bfloat16
    grads = (H.grad_buffers(numels, gdt), H.grad_buffers(numels, gdt), H.grad_buffers(numels, gdt))
    return dev, ctx, orc, grads


# ---------------------------------------------------------------------------------------------
# config 1: plain-GD quadratic surrogate, P = 2^20, eta = 0.1, K = 4, 20 active steps
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("alpha", [1.0, 0.5])
def test_surrogate_config1_lockstep_and_closed_form(fused, alpha):
    P, eta, K = 1 << 20, 0.1, 4
    problem = synth.surrogate_problem(P, 0, device="cuda")
    cfg = B.make_config(optimizer="gd", K=K, alpha=alpha, delta=0.0, lr=eta, fuse_step2=fused, tau=3.0, window=10)
    dev, ctx, orc, grads = build([P], cfg, problem)
    grad_fn = quad_trainer(problem, [P])
    h, ts, th0 = (H.f64(x) for x in (problem.h, problem.theta_star, problem.theta_0))
    rho = 1.0 - eta * h
    for step in range(20):
        start = dev.host("theta")[0]
        info, _ = H.lockstep_active_step(ctx, dev, orc, grad_fn, grads, dtol=1e-5, fused=fused, what=f"step {step}")
        assert not info.tripped
        # one outer step multiplies the error by rho (1 - alpha + alpha rho^K); alpha = 1: K + 1 GD steps
        want = ts + rho * (1 - alpha + alpha * rho ** K) * (start - ts)
        got = dev.host("theta")[0]
        assert np.linalg.norm(got - want) <= 1e-5 * np.linalg.norm(want - start) + 6 * 2.0 ** -24 * np.linalg.norm(want)
    st = B.gxpo_get_state(ctx)
    assert (st.t, st.optim_steps, st.backward_passes, st.s_star) == (20, 60, 60, -1)
    # free-running closed form: theta_20 = theta* + [rho (1 - alpha + alpha rho^K)]^20 (theta_0 - theta*)
    want = ts + (rho * (1 - alpha + alpha * rho ** K)) ** 20 * (th0 - ts)
    H.assert_close(dev.host("theta")[0], want, "theta_20 closed form", rtol=1e-5)


# ---------------------------------------------------------------------------------------------
# config 2 shape at reduced size: AdamW, noisy quadratic, K = 8, ragged multi-tensor
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("fused,alternating", [(True, False), (False, False), (True, True)])
@pytest.mark.parametrize("grad_dtype", ["f32", "bf16"])
def test_adamw_ragged_lockstep(fused, alternating, grad_dtype):
    numels = RAGGED
    P = sum(numels)
    problem = synth.policy_problem(P, seed=1, sigma=0.05, device="cuda")
    cfg = B.make_config(optimizer="adamw", grad_dtype=grad_dtype, K=8, alpha=0.5, delta=1.75e-3, lr=1e-6,
                        weight_decay=0.01, fuse_step2=fused, tau=3.0, window=10, gate_min_count=2,
                        copy_mask=7)
    dev, ctx, orc, grads = build(numels, cfg, problem, with_copy=True, alternating=alternating)
    step_id = [0]
    noise = lambda: synth.step_noise(problem, step_id[0])
    grad_fn = quad_trainer(problem, numels, step_noise=noise)
    for step in range(4):
        step_id[0] = step
        H.lockstep_active_step(ctx, dev, orc, grad_fn, grads, dtol=1e-4, fused=fused, check_copy=True,
                               what=f"{grad_dtype} fused={fused} alternating={alternating} step {step}")
    st = B.gxpo_get_state(ctx)
    assert (st.t, st.optim_steps, st.backward_passes) == (4, 12, 12)
    dev.check_canaries()


@pytest.mark.parametrize("grad_dtype", ["f32", "bf16"])
def test_thousands_of_tiny_tensors(grad_dtype):
    """1500 tensors of 1 .. 700 elements: almost every block is a ragged tail and the block -> tensor
    search walks up to 64 table entries per block; per-tensor norms are checked one by one."""
    rng = np.random.default_rng(31)
    numels = [int(x) for x in rng.integers(1, 700, size=1500)]
    problem = synth.policy_problem(sum(numels), seed=31, sigma=0.05, device="cuda")
    cfg = B.make_config(grad_dtype=grad_dtype, K=5, alpha=0.5, delta=1.75e-3, lr=1e-4, weight_decay=0.01, gate_min_count=2,
                        copy_mask=7, diagnostics=True)
    dev, ctx, orc, grads = build(numels, cfg, problem, with_copy=True)
    step_id = [0]
    grad_fn = quad_trainer(problem, numels, step_noise=lambda: synth.step_noise(problem, step_id[0]))
    for step in range(2):
        step_id[0] = step
        H.lockstep_active_step(ctx, dev, orc, grad_fn, grads, dtol=1e-4, fused=True, check_copy=True, what=f"tiny tensors step {step}")
    got, want = B.gxpo_tensor_norms(ctx), orc.tensor_norms()
    assert len(got) == 1500
    np.testing.assert_allclose(got, want, rtol=1e-12)
    dev.check_canaries()


@pytest.mark.parametrize("fused", [True, False])
def test_lockstep_on_a_side_stream(fused):
    """Every call takes the caller's stream: run a whole active step, with clipping and
    diagnostics so that every kernel and both host read-backs are involved, on a
    non-default stream (default priority) while the default stream stays idle."""
    numels = [4099, 257, 70001]
    problem = synth.policy_problem(sum(numels), seed=9, sigma=0.05, device="cuda")
    cfg = B.make_config(K=8, alpha=0.5, delta=1.75e-3, lr=1e-4, weight_decay=0.01, fuse_step2=fused, gate_min_count=2,
                        diagnostics=1, clip_norm=5.0)
    dev, ctx, orc, grads = build(numels, cfg, problem)
    step_id = [0]
    grad_fn = quad_trainer(problem, numels, step_noise=lambda: synth.step_noise(problem, step_id[0]))
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        assert torch.cuda.current_stream().cuda_stream == side.cuda_stream != 0
        for step in range(3):
            step_id[0] = step
            H.lockstep_active_step(ctx, dev, orc, grad_fn, grads, dtol=1e-4, fused=fused, what=f"side stream step {step}")
        side.synchronize()
    assert B.gxpo_get_state(ctx).t == 3


@pytest.mark.parametrize("K", [2, 3, 5, 10])
@pytest.mark.parametrize("alpha", [0.0, 0.1, 0.5, 1.0])
def test_paper_K_alpha_grid(K, alpha):
    numels = [70001, 513]
    problem = synth.policy_problem(sum(numels), seed=5, sigma=0.05, device="cuda")
    cfg = B.make_config(K=K, alpha=alpha, delta=1.75e-3, lr=1e-4, gate_min_count=2)
    dev, ctx, orc, grads = build(numels, cfg, problem)
    step_id = [0]
    grad_fn = quad_trainer(problem, numels, step_noise=lambda: synth.step_noise(problem, step_id[0]))
    for step in range(2):
        step_id[0] = step
        H.lockstep_active_step(ctx, dev, orc, grad_fn, grads, dtol=1e-4, fused=True, what=f"K={K} alpha={alpha}")
    if alpha == 0.0:
        pass  # theta~ == theta^t is implied by the oracle comparison


# ---------------------------------------------------------------------------------------------
# the extrapolation factor itself, at full fp32 resolution: theta^t = 0, theta^{t,1} = 1
# ---------------------------------------------------------------------------------------------
def crafted_gradient_pairs(delta32: float):
    rng = np.random.default_rng(11)
    g0, g1 = [], []

    def add(a, b):
        g0.append(np.float32(a)); g1.append(np.float32(b))
    for base in (1.0, -0.37, 3.5e-3, 11.0):
        add(base, base)                                    # r = 1 exactly
        add(base, 0.0)                                     # r = 0
        add(base, -base)                                   # r = -1 exactly: degenerate
        for eps in (2.0 ** -23, 2.0 ** -20, 1e-6, 1e-4, 1e-2, 0.3):
            add(base, base * (1 + eps)); add(base, base * (1 - eps))          # around +1
            add(base, -base * (1 + eps)); add(base, -base * (1 - eps))        # around the pole at -1
        for r in (0.5, -0.5, 2.0, -2.0, 3.0, -3.0, 10.0, -7.0, 1e-3):
            add(base, base * r)
    d = np.float32(delta32)
    add(d, d); add(-d, d)                                  # |g0| == delta: inactive
    add(np.nextafter(d, np.float32(1)), d)                 # one ulp above: active
    add(np.nextafter(d, np.float32(0)), 5.0)               # one ulp below: inactive
    add(0.0, 1.0); add(-0.0, -1.0)                         # zero gradient never forms a ratio
    a = rng.normal(size=4000).astype(np.float32); b = rng.normal(size=4000).astype(np.float32)
    g0 += list(a); g1 += list(b)                           # heavy-tailed ratios
    a = rng.normal(size=4000).astype(np.float32)
    g0 += list(a); g1 += list((a * (1 + 1e-3 * rng.normal(size=4000))).astype(np.float32))   # r ~ 1, the common case
    return np.array(g0, dtype=np.float32), np.array(g1, dtype=np.float32)


@pytest.mark.parametrize("K", [2, 3, 4, 5, 8, 9, 10])
@pytest.mark.parametrize("r_max", [math.inf, 4.0, 1.0])
@pytest.mark.parametrize("fused", [True, False])
def test_scale_factor_crafted(K, r_max, fused):
    check_scale_factor(K, r_max, fused)


@pytest.mark.parametrize("K", [64, 65, 129])
@pytest.mark.parametrize("fused", [True, False])
def test_scale_factor_long_horizons(K, fused):
    """Horizons far beyond the paper's K <= 10, with |r| clamped to 1 so that neither side overflows:
    the series loop runs K/2 times; its rounding error grows like K 2^-24, still inside 1e-5 here."""
    check_scale_factor(K, 1.0, fused)


def check_scale_factor(K, r_max, fused):
    delta = 1e-3
    g0_np, g1_np = crafted_gradient_pairs(float(np.float32(delta)))
    n = g0_np.size
    lr = 2.0 ** -10
    alpha = 1.0
    cfg = B.make_config(optimizer="gd", K=K, alpha=alpha, delta=delta, r_max=r_max, lr=lr, fuse_step2=fused)
    dev = H.DeviceState([n], adam=False, with_copy=False)
    dev.views["theta"][0].zero_()
    ctx = B.gxpo_init(cfg, dev.tensor_dicts())
    g0 = torch.from_numpy(g0_np).cuda()
    g1 = torch.from_numpy(g1_np).cuda()
    B.gxpo_fast_steps(ctx, 0, [g0])
    if not fused:
        # the buffers are the caller's: plant theta^{t,2} = 1, so that theta~ = alpha * scale exactly
        B.gxpo_fast_steps(ctx, 1, [g1])
        dev.views["theta_probe"][0].fill_(1.0)
    else:
        # fused: theta^{t,2} - theta^t = -lr (g0 + g1) is formed in registers; lr is a power of two, so the
        # products are exact and the sum is rounded once from exact inputs, even where g0 + g1 cancels
        B.gxpo_fast_steps(ctx, 1, [g1])
    B.gxpo_extrapolate(ctx, [g0], [g1])
    torch.cuda.synchronize()
    got = dev.host("theta")[0]
    g0d, g1d = g0_np.astype(np.float64), g1_np.astype(np.float64)
    th2 = (-lr * (g0d + g1d)) if fused else np.ones(n)
    scale, _, want = O.extrapolate(np.zeros(n), th2, g0d, g1d, K, alpha, delta, r_max)
    finite = np.isfinite(want) & (np.abs(want) < 1e30)
    assert finite.sum() > 0.9 * n
    rel = np.abs(got[finite] - want[finite]) / np.maximum(np.abs(want[finite]), 1e-30)
    rel[(want[finite] == 0.0) & (got[finite] == 0.0)] = 0.0
    worst = int(np.argmax(rel))
    assert rel.max() <= 1e-5, (f"scale mismatch: rel {rel.max():.3e} at g0={g0_np[finite][worst]!r} g1={g1_np[finite][worst]!r} "
                               f"got {got[finite][worst]!r} want {want[finite][worst]!r}")
    # special values survive fp32 exactly
    same = (g0_np == g1_np) & (np.abs(g0_np) > np.float32(delta))
    assert same.any()
    np.testing.assert_allclose(got[same], th2[same] * (K / 2), rtol=2e-7)
    degenerate = (g1_np == -g0_np) | ~(np.abs(g0_np) > np.float32(delta))
    np.testing.assert_allclose(got[degenerate], th2[degenerate], rtol=2e-7)


# ---------------------------------------------------------------------------------------------
# partly fresh noise between the probes: broad, Cauchy-tailed retention ratios, clamped
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("K", [5, 8])
def test_broad_retention_spread_with_clamp(K):
    numels = [50000, 7777]
    P = sum(numels)
    problem = synth.policy_problem(P, seed=7, sigma=0.05, device="cuda")
    cfg = B.make_config(K=K, alpha=0.5, delta=1.75e-3, r_max=2.0, lr=1e-4, gate_min_count=2)
    dev, ctx, orc, grads = build(numels, cfg, problem)
    call = [0]

    def noise():
        base = synth.step_noise(problem, 100)
        fresh = synth.step_noise(problem, 200 + call[0])
        call[0] += 1
        return 0.5 * base + math.sqrt(0.75) * fresh
    grad_fn = quad_trainer(problem, numels, step_noise=noise)
    H.lockstep_active_step(ctx, dev, orc, grad_fn, grads, dtol=1e-4, fused=True, what="broad r")
    r = H.f64(grads[1][0]) / H.f64(grads[0][0])
    assert np.std(np.clip(r, -5, 5)) > 0.5              # the ratios really are broad


# ---------------------------------------------------------------------------------------------
# mechanism diagnostics (appendix table of active-phase diagnostics), fused into the passes
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("grad_dtype", ["f32", "bf16"])
def test_mechanism_diagnostics_policy_like(fused, grad_dtype):
    numels = RAGGED
    problem = synth.policy_problem(sum(numels), seed=21, sigma=0.05, device="cuda")
    cfg = B.make_config(grad_dtype=grad_dtype, K=5, alpha=0.5, delta=1.75e-3, lr=1e-4, fuse_step2=fused, gate_min_count=2,
                        diagnostics=True)
    dev, ctx, orc, grads = build(numels, cfg, problem)
    step_id = [0]
    grad_fn = quad_trainer(problem, numels, step_noise=lambda: synth.step_noise(problem, step_id[0]))
    with pytest.raises(B.GxpoError):
        B.gxpo_get_diagnostics(ctx)                      # nothing to report yet
    for step in range(3):
        step_id[0] = step
        H.lockstep_active_step(ctx, dev, orc, grad_fn, grads, dtol=1e-4, fused=fused, what=f"diag step {step}")
    d = B.gxpo_get_diagnostics(ctx)
    assert d.t == 2 and 0.01 < d.inactive_fraction < 0.06 and 0.9 < d.cos_g0_g_slow <= 1.0
    # the trainer may hand g_slow in in g0's buffers; the cosine is then reported as NaN
    H.lockstep_active_step(ctx, dev, orc, grad_fn, (grads[0], grads[1], grads[0]), dtol=1e-4, fused=fused, what="aliased")


@pytest.mark.parametrize("fused", [True, False])
def test_mechanism_diagnostics_ignore_lanes_past_a_ragged_end(fused):
    """With adam_eps = 0 a lane past the end of a tensor (all-zero loads) computes 0/0 in its
    would-be AdamW step; nothing of it may reach the displacement sums."""
    numels = [1, 3, 255, 257, 1000, 4099]
    problem = synth.policy_problem(sum(numels), seed=23, sigma=0.05, device="cuda")
    cfg = B.make_config(K=5, alpha=0.5, delta=1.75e-3, lr=1e-4, adam_eps=0.0, fuse_step2=fused, gate_min_count=2, diagnostics=True)
    dev, ctx, orc, grads = build(numels, cfg, problem)
    grad_fn = quad_trainer(problem, numels, step_noise=lambda: synth.step_noise(problem, 0))
    H.lockstep_active_step(ctx, dev, orc, grad_fn, grads, dtol=1e-4, fused=fused, what="eps = 0 ragged diagnostics")
    d = B.gxpo_get_diagnostics(ctx)
    assert math.isfinite(d.displacement_ratio) and d.displacement_ratio > 1.0


def test_mechanism_diagnostics_broad_ratios_and_surrogate():
    # broad, clamped ratios
    numels = [60000, 333]
    problem = synth.policy_problem(sum(numels), seed=22, sigma=0.05, device="cuda")
    cfg = B.make_config(K=4, alpha=0.5, delta=1.75e-3, r_max=2.0, lr=1e-4, gate_min_count=2, diagnostics=True)
    dev, ctx, orc, grads = build(numels, cfg, problem)
    call = [0]

    def noise():
        call[0] += 1
        return 0.5 * synth.step_noise(problem, 100) + math.sqrt(0.75) * synth.step_noise(problem, 200 + call[0])
    H.lockstep_active_step(ctx, dev, orc, quad_trainer(problem, numels, step_noise=noise), grads, dtol=1e-4, fused=True, what="broad")
    d = B.gxpo_get_diagnostics(ctx)
    assert d.retention_std > 0.5
    # plain-GD surrogate: every statistic has a closed form (r_i = 1 - eta h_i)
    P, eta, K = 1 << 18, 0.1, 4
    problem = synth.surrogate_problem(P, 0, device="cuda")
    cfg = B.make_config(optimizer="gd", K=K, alpha=1.0, delta=0.0, lr=eta, diagnostics=True)
    dev, ctx, orc, grads = build([P], cfg, problem)
    H.lockstep_active_step(ctx, dev, orc, quad_trainer(problem, [P]), grads, dtol=1e-5, fused=True, what="surrogate diag")
    d = B.gxpo_get_diagnostics(ctx)
    rho = 1 - eta * H.f64(problem.h)
    S = lambda n: sum(rho ** j for j in range(n))
    assert d.retention_mean == pytest.approx(float(np.mean(rho)), rel=1e-6)
    assert d.retention_std == pytest.approx(float(np.std(rho)), rel=1e-5)
    assert d.scale_mean == pytest.approx(float(np.mean(S(K) / S(2))), rel=1e-6)
    assert d.inactive_fraction == 0.0


def test_diagnostics_are_refused_without_the_flag():
    problem = synth.policy_problem(1000, seed=3, device="cuda")
    dev, ctx, orc, grads = build([1000], B.make_config(), problem)
    with pytest.raises(B.GxpoError) as e:
        B.gxpo_get_diagnostics(ctx)
    assert e.value.code == B.GXPO_ERR_BAD_STATE


# ---------------------------------------------------------------------------------------------
# global-norm gradient clipping (the paper trains with clipping at 1.0)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("grad_dtype", ["f32", "bf16"])
def test_gradient_clipping_lockstep(fused, grad_dtype):
    numels = RAGGED
    problem = synth.policy_problem(sum(numels), seed=31, sigma=0.05, device="cuda")
    # ||g|| is about 0.05 * sqrt(P) = 26 here: clip_norm = 20 clips the sigma = 0.05 gradients, not the sigma = 0.03 ones
    cfg = B.make_config(grad_dtype=grad_dtype, K=5, alpha=0.5, delta=1.75e-3, lr=1e-4, fuse_step2=fused, gate_min_count=2,
                        clip_norm=20.0, diagnostics=True)
    dev, ctx, orc, grads = build(numels, cfg, problem)
    step_id, call = [0], [0]
    sigmas = [0.05, 0.03, 0.05,   0.03, 0.05, 0.03,   0.05, 0.05, 0.05]

    def grad_fn(thetas, outs):
        inner = quad_trainer(problem, numels, sigma=sigmas[call[0]], step_noise=lambda: synth.step_noise(problem, step_id[0]))
        call[0] += 1
        inner(thetas, outs)
    for step in range(3):
        step_id[0] = step
        info, _ = H.lockstep_active_step(ctx, dev, orc, grad_fn, grads, dtol=1e-4, fused=fused, what=f"clip step {step}")
    assert info.norm > 20.0                                # the gate sees the norm before clipping
    # and the fallback step clips too
    st = B.gxpo_get_state(ctx); st.s_star = st.t; B.gxpo_set_state(ctx, st)
    H.sync_oracle_to_device(orc, dev, st.optim_steps)
    orc.gate.s_star = orc.t = int(st.t)
    call[0] = 0
    grad_fn(dev.views["theta"], grads[0])
    B.gxpo_fallback_step(ctx, grads[0])
    ref = orc.fallback_step([H.f64(g) for g in grads[0]])
    for i in range(len(numels)):
        H.assert_close(dev.host("theta")[i], ref[i], f"clipped fallback theta tensor {i}")
        H.assert_close(dev.host("v")[i], orc.v[i], f"clipped fallback v tensor {i}")


def test_inactive_clipping_changes_nothing():
    numels = [50000, 77]
    problem = synth.policy_problem(sum(numels), seed=32, sigma=0.05, device="cuda")
    outs = []
    for clip in (0.0, 1e9):
        cfg = B.make_config(K=8, lr=1e-4, delta=1.75e-3, clip_norm=clip, gate_min_count=2)
        dev, ctx, orc, grads = build(numels, cfg, problem)
        grad_fn = quad_trainer(problem, numels, step_noise=lambda: synth.step_noise(problem, 0))
        info, _ = H.lockstep_active_step(ctx, dev, orc, grad_fn, grads, dtol=1e-4, fused=True, what=f"clip={clip}")
        outs.append((info.norm, [x.clone() for x in dev.views["theta"]], [x.clone() for x in dev.views["v"]]))
    assert outs[0][0] == outs[1][0]
    for a, b in zip(outs[0][1] + outs[0][2], outs[1][1] + outs[1][2]):
        assert torch.equal(a, b)


# ---------------------------------------------------------------------------------------------
# explicit lookahead: n real fast steps, reposition, slow correction (the scheme the paper compares with)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n_steps,grad_dtype,clip", [(3, "f32", 0.0), (5, "bf16", 0.0), (2, "f32", 20.0)])
def test_explicit_lookahead_lockstep(n_steps, grad_dtype, clip):
    numels = RAGGED
    problem = synth.policy_problem(sum(numels), seed=41, sigma=0.05, device="cuda")
    cfg = B.make_config(grad_dtype=grad_dtype, alpha=0.5, lr=1e-4, explicit_steps=n_steps, clip_norm=clip, gate_min_count=2,
                        copy_mask=7)
    dev, ctx, orc, grads = build(numels, cfg, problem, with_copy=True)
    g_fast, _, g_slow = grads
    for step in range(3):
        noise = synth.step_noise(problem, step)
        grad_fn = quad_trainer(problem, numels, step_noise=lambda: noise)
        st = B.gxpo_get_state(ctx)
        H.sync_oracle_to_device(orc, dev, st.optim_steps)
        start = dev.host("theta")
        src = dev.views["theta"]
        for j in range(n_steps):
            grad_fn(src, g_fast)
            with pytest.raises(B.GxpoError):
                B.gxpo_fast_steps(ctx, j + 1 if j + 1 < n_steps else 0, g_fast)        # out of order
            B.gxpo_fast_steps(ctx, j, g_fast)
            ref = orc.explicit_fast_step(j, [H.f64(g) for g in g_fast])
            src = dev.views["theta_probe"]
            for i in range(len(numels)):
                H.assert_close(dev.host("theta_probe")[i], ref[i], f"explicit step {j} tensor {i}")
                H.assert_close(dev.host("v")[i], orc.v[i], f"explicit step {j} v tensor {i}")
            H.check_bf16_copy_of(dev, "theta_probe", ref, f"explicit step {j}")
        B.gxpo_extrapolate(ctx)
        ref_t = orc.explicit_reposition()
        num = den = 0.0
        for i in range(len(numels)):
            got = dev.host("theta")[i]
            H.assert_close(got, ref_t[i], f"explicit theta~ tensor {i}")
            num += float(np.sum(((got - start[i]) - (ref_t[i] - start[i])) ** 2)); den += float(np.sum((ref_t[i] - start[i]) ** 2))
        assert math.sqrt(num) <= 1e-4 * math.sqrt(den) + (2 + n_steps) * 2.0 ** -24 * math.sqrt(sum(float(np.sum(r * r)) for r in ref_t))
        grad_fn(dev.views["theta"], g_slow)
        B.gxpo_slow_step(ctx, g_slow)
        ref_n = orc.slow_step([H.f64(g) for g in g_slow])
        info, ref_info = B.gxpo_gate(ctx), orc.gate_step()
        for i in range(len(numels)):
            H.assert_close(dev.host("theta")[i], ref_n[i], f"explicit theta^(t+1) tensor {i}")
        assert info.norm == pytest.approx(ref_info.norm, rel=1e-12) and bool(info.tripped) == ref_info.tripped
        dev.check_canaries()
    st = B.gxpo_get_state(ctx)
    assert st.backward_passes == orc.backward_passes == 3 * (n_steps + 1) and st.optim_steps == 3 * (n_steps + 1)


def test_explicit_lookahead_matches_extrapolation_on_the_surrogate():
    """Plain GD on the diagonal quadratic: K real fast steps and the 3-pass extrapolation reach the same theta~."""
    P, eta, K = 1 << 18, 0.1, 5
    problem = synth.surrogate_problem(P, 0, device="cuda")
    outs = []
    for explicit in (0, K):
        cfg = B.make_config(optimizer="gd", K=K, alpha=1.0, delta=0.0, lr=eta, explicit_steps=explicit)
        dev, ctx, orc, grads = build([P], cfg, problem)
        grad_fn = quad_trainer(problem, [P])
        g = grads[0]
        if explicit:
            src = dev.views["theta"]
            for j in range(K):
                grad_fn(src, g); B.gxpo_fast_steps(ctx, j, g); src = dev.views["theta_probe"]
            B.gxpo_extrapolate(ctx)
        else:
            grad_fn(dev.views["theta"], grads[0]); B.gxpo_fast_steps(ctx, 0, grads[0])
            grad_fn(dev.views["theta_probe"], grads[1]); B.gxpo_fast_steps(ctx, 1, grads[1])
            B.gxpo_extrapolate(ctx, grads[0], grads[1])
        outs.append(dev.host("theta")[0])
    start = H.f64(problem.theta_0)
    assert np.linalg.norm(outs[0] - outs[1]) <= 2e-6 * np.linalg.norm(outs[1] - start)


# ---------------------------------------------------------------------------------------------
# gate transition and fallback (config 5 at reduced size)
# ---------------------------------------------------------------------------------------------
def test_gate_transition_free_running_and_fallback():
    """50 free-running steps, sigma raised from 0.05 to 1.0 at step 30.  GPU and oracle
    each follow their own trajectory (own parameters, own gradients of the same loss and
    noise); every gate decision must agree.  With w = 10 a stationary norm sequence trips
    tau = 3 by chance about once in a hundred steps; if that happens before step 30 both
    sides must agree on it, and both are then put back into the active phase through the
    state interface so that the real transition at step 30 is still exercised."""
    P = (1 << 18) + 37
    numels = [P]
    problem = synth.policy_problem(P, seed=4, sigma=0.05, device="cuda")
    cfg = B.make_config(K=8, alpha=0.5, delta=1.75e-3, lr=1e-6, tau=3.0, window=10)
    dev, ctx, orc, grads = build(numels, cfg, problem)
    g0b, g1b, gsb = grads
    h64, ts64 = H.f64(problem.h), H.f64(problem.theta_star)
    sigma_of = lambda step: 0.05 if step < 30 else 1.0
    early_trips, n_active = [], 0
    for step in range(50):
        xi = synth.step_noise(problem, step)
        xi64 = H.f64(xi)
        sig = sigma_of(step)
        gpu_grad = lambda th, out: out[0].copy_(synth.quadratic_grad(problem, th[0], xi, sig))
        # the oracle's trainer evaluates the same loss at the oracle's own fp64 parameters,
        # and hands the gradient over in fp32 like the GPU's trainer does
        ref_grad = lambda ths: [(h64 * (ths[0] - ts64) + sig * xi64).astype(np.float32).astype(np.float64)]
        st = B.gxpo_get_state(ctx)
        active_gpu = st.s_star < 0 or st.t < st.s_star
        assert active_gpu == orc.is_active(), f"phase differs at step {step}"
        if active_gpu:
            n_active += 1
            gpu_grad(dev.views["theta"], g0b); B.gxpo_fast_steps(ctx, 0, g0b)
            gpu_grad(dev.views["theta_probe"], g1b); B.gxpo_fast_steps(ctx, 1, g1b)
            B.gxpo_extrapolate(ctx, g0b, g1b)
            gpu_grad(dev.views["theta"], gsb); B.gxpo_slow_step(ctx, gsb)
            info = B.gxpo_gate(ctx)
            ref = orc.train_step(ref_grad)
            assert bool(info.evaluated) == ref.evaluated
            assert bool(info.tripped) == ref.tripped, f"gate decision differs at step {step}: Z {info.z} vs {ref.z}"
            assert info.norm == pytest.approx(ref.norm, rel=1e-6)
            if ref.evaluated:
                assert info.z == pytest.approx(ref.z, rel=1e-3, abs=1e-2)
            if info.tripped:
                assert info.s_star == ref.s_star == step + 1
                if step < 30:                                  # chance trip: agree, then re-arm both sides
                    early_trips.append(step)
                    st = B.gxpo_get_state(ctx)
                    st.s_star = -1
                    B.gxpo_set_state(ctx, st)
                    orc.gate.s_star = None
        else:
            with pytest.raises(B.GxpoError) as e:
                B.gxpo_fast_steps(ctx, 0, g0b)
            assert e.value.code == B.GXPO_ERR_BAD_STATE
            gpu_grad(dev.views["theta"], g0b); B.gxpo_fallback_step(ctx, g0b)
            orc.train_step(ref_grad)
    print("chance trips before the transition:", early_trips)
    st = B.gxpo_get_state(ctx)
    assert st.s_star == 31 and orc.s_star == 31 and st.t == 50     # first sigma = 1 step is t = 30
    assert n_active == 31
    assert st.backward_passes == orc.backward_passes == 3 * 31 + (50 - 31)
    assert st.optim_steps == orc.optim_steps
    H.assert_close(dev.host("theta")[0], orc.theta[0], "theta after 50 free-running steps")
    H.assert_close(dev.host("m")[0], orc.m[0], "m after 50 steps")
    H.assert_close(dev.host("v")[0], orc.v[0], "v after 50 steps")
    dev.check_canaries()


@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("grad_dtype", ["f32", "bf16"])
def test_fallback_step_parity_and_bitwise_equal_to_first_fast_step(grad_dtype, fused):
    numels = RAGGED
    P = sum(numels)
    problem = synth.policy_problem(P, seed=9, sigma=0.05, device="cuda")
    cfg = B.make_config(grad_dtype=grad_dtype, lr=1e-6, copy_mask=7, fuse_step2=fused)
    dev_a, ctx_a, orc, grads = build(numels, cfg, problem, with_copy=True)
    dev_b, ctx_b, _, _ = build(numels, cfg, problem, with_copy=True)
    g0b = grads[0]
    grad_fn = quad_trainer(problem, numels, step_noise=lambda: synth.step_noise(problem, 0))
    # warm both contexts up with one identical active step so the moments are non-trivial
    for ctx, dev in ((ctx_a, dev_a), (ctx_b, dev_b)):
        grad_fn(dev.views["theta"], g0b)
        g1b = grads[1]
        for a, b in zip(g1b, g0b):
            a.copy_(b)
        B.gxpo_fast_steps(ctx, 0, g0b); B.gxpo_fast_steps(ctx, 1, g1b); B.gxpo_extrapolate(ctx, g0b, g1b)
        B.gxpo_slow_step(ctx, g0b); B.gxpo_gate(ctx)
    for k in ("theta", "m", "v"):
        for a, b in zip(dev_a.views[k], dev_b.views[k]):
            assert torch.equal(a, b)
    # fallback is refused before the gate trips
    with pytest.raises(B.GxpoError) as e:
        B.gxpo_fallback_step(ctx_a, g0b)
    assert e.value.code == B.GXPO_ERR_BAD_STATE
    st = B.gxpo_get_state(ctx_a)
    st.s_star = st.t                                    # restore a tripped state
    B.gxpo_set_state(ctx_a, st)
    H.sync_oracle_to_device(orc, dev_a, st.optim_steps)
    orc.gate.s_star = orc.t = int(st.t)
    start = dev_a.host("theta")
    m_before = [x.clone() for x in dev_b.views["m"]]
    grad_fn(dev_a.views["theta"], g0b)
    B.gxpo_fallback_step(ctx_a, g0b)                    # theta <- OptimStep(theta, g0), in place
    B.gxpo_fast_steps(ctx_b, 0, g0b)                    # theta_probe <- OptimStep(theta, g0)
    torch.cuda.synchronize()
    ref = orc.fallback_step([H.f64(g) for g in g0b])
    for i in range(len(numels)):
        H.assert_close(dev_a.host("theta")[i], ref[i], f"fallback theta tensor {i}")
        H.assert_close(dev_a.host("m")[i], orc.m[i], f"fallback m tensor {i}")
        H.assert_close(dev_a.host("v")[i], orc.v[i], f"fallback v tensor {i}")
        assert torch.equal(dev_a.views["theta"][i], dev_b.views["theta_probe"][i])      # same arithmetic, bit for bit
        if fused:       # the probe pass of the fused schedule leaves the stored moments alone
            assert torch.equal(dev_b.views["m"][i], m_before[i])
        else:
            assert torch.equal(dev_a.views["m"][i], dev_b.views["m"][i])
            assert torch.equal(dev_a.views["v"][i], dev_b.views["v"][i])
    num = math.sqrt(sum(float(np.sum(((g - s) - (r - s)) ** 2)) for g, r, s in zip(dev_a.host("theta"), ref, start)))
    den = math.sqrt(sum(float(np.sum((r - s) ** 2)) for r, s in zip(ref, start)))
    ref_norm = math.sqrt(sum(float(np.sum(r * r)) for r in ref))
    assert num <= 1e-4 * den + 2.0 ** -24 * ref_norm
    H.check_bf16_copy(dev_a, ref, "fallback")
    st2 = B.gxpo_get_state(ctx_a)
    assert (st2.t, st2.optim_steps, st2.backward_passes) == (st.t + 1, st.optim_steps + 1, st.backward_passes + 1)
    dev_a.check_canaries(); dev_b.check_canaries()


# ---------------------------------------------------------------------------------------------
# call order, errors, state round trip
# ---------------------------------------------------------------------------------------------
def test_call_order_state_machine_and_errors():
    n = 1000
    problem = synth.policy_problem(n, seed=3, device="cuda")
    cfg = B.make_config(fuse_step2=True)
    dev, ctx, orc, grads = build([n], cfg, problem)
    g = [torch.randn(n, device="cuda")]
    g_other = [torch.randn(n, device="cuda")]

    def refused(fn, code=B.GXPO_ERR_BAD_STATE):
        with pytest.raises(B.GxpoError) as e:
            fn()
        assert e.value.code == code and e.value.message
    refused(lambda: B.gxpo_fast_steps(ctx, 1, g))
    refused(lambda: B.gxpo_extrapolate(ctx, g, g))
    refused(lambda: B.gxpo_slow_step(ctx, g))
    refused(lambda: B.gxpo_gate(ctx))
    refused(lambda: B.gxpo_fallback_step(ctx, g))
    refused(lambda: B.gxpo_tensor_norms(ctx))
    refused(lambda: B.gxpo_fast_steps(ctx, 2, g), B.GXPO_ERR_INVALID_ARG)
    B.gxpo_fast_steps(ctx, 0, g)
    refused(lambda: B.gxpo_fast_steps(ctx, 0, g))
    refused(lambda: B.gxpo_set_state(ctx, B.gxpo_get_state(ctx)))
    refused(lambda: B.gxpo_fast_steps(ctx, 1, g), B.GXPO_ERR_INVALID_ARG)          # g1 written over g0
    refused(lambda: B.gxpo_fast_steps(ctx, 1, dev.views["theta"]), B.GXPO_ERR_INVALID_ARG)   # a gradient inside an engine buffer
    g1 = [torch.randn(n, device="cuda")]
    B.gxpo_fast_steps(ctx, 1, g1)
    refused(lambda: B.gxpo_extrapolate(ctx, g, g_other), B.GXPO_ERR_INVALID_ARG)   # not the g1 that was recorded
    refused(lambda: B.gxpo_extrapolate(ctx, g_other, g1), B.GXPO_ERR_INVALID_ARG)  # not the g0 the probe pass used
    B.gxpo_extrapolate(ctx, g, g1)
    refused(lambda: B.gxpo_fast_steps(ctx, 0, g))
    B.gxpo_slow_step(ctx, g)
    refused(lambda: B.gxpo_slow_step(ctx, g))
    info = B.gxpo_gate(ctx)
    assert info.t == 0 and not info.evaluated and info.norm == pytest.approx(float(g[0].double().norm()), rel=1e-12)
    # misaligned / foreign gradient pointers
    bad = [torch.randn(n + 1, device="cuda")[1:]]
    refused(lambda: B.gxpo_fast_steps(ctx, 0, bad), B.GXPO_ERR_ALIGNMENT)
    with pytest.raises(ValueError):
        B.gxpo_fast_steps(ctx, 0, [torch.randn(n, device="cuda", dtype=torch.float64)])
    # state round trip
    st = B.gxpo_get_state(ctx)
    assert (st.t, st.optim_steps, st.backward_passes, st.window_len, st.phase) == (1, 3, 3, 1, B.GXPO_PHASE_IDLE)
    st.t, st.optim_steps, st.s_star = 7, 21, 9
    B.gxpo_set_state(ctx, st)
    st2 = B.gxpo_get_state(ctx)
    assert (st2.t, st2.optim_steps, st2.s_star) == (7, 21, 9)
    B.gxpo_fast_steps(ctx, 0, g)                       # still active: t = 7 < s* = 9
    B.gxpo_destroy(ctx)


@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("optimizer,numels", [("adamw", RAGGED), ("adamw", [70001]), ("gd", [257, 4099, 5])])
def test_parameter_groups_lockstep(fused, optimizer, numels):
    """Per-tensor lr / weight-decay multipliers (no decay on some tensors, a lower or zero learning rate on
    others), on the ragged list, on a single flat tensor (pointers and multipliers from the kernel
    arguments) and with plain GD."""
    problem = synth.policy_problem(sum(numels), seed=15, sigma=0.05, device="cuda")
    cfg = B.make_config(optimizer=optimizer, K=5, alpha=0.5, delta=1.75e-3, lr=1e-4, weight_decay=0.1, fuse_step2=fused,
                        gate_min_count=2, tau=1e6)
    dev, ctx, orc, grads = build(numels, cfg, problem)
    pattern_lr, pattern_wd = [1.0, 0.25, 1.0, 0.0, 3.0], [1.0, 0.0, 2.0, 1.0, 0.5]
    lr_scale = [pattern_lr[i % 5] for i in range(len(numels))] if len(numels) > 1 else [0.5]
    wd_scale = [pattern_wd[i % 5] for i in range(len(numels))] if len(numels) > 1 else [0.0]
    B.gxpo_set_tensor_options(ctx, lr_scale, wd_scale)
    orc.lr_scale, orc.weight_decay_scale = list(lr_scale), list(wd_scale)
    step_id = [0]
    grad_fn = quad_trainer(problem, numels, step_noise=lambda: synth.step_noise(problem, step_id[0]))
    before = dev.host("theta")
    for step in range(3):
        step_id[0] = step
        H.lockstep_active_step(ctx, dev, orc, grad_fn, grads, dtol=1e-4, fused=fused, what=f"groups step {step}")
    after = dev.host("theta")
    for i, a in enumerate(lr_scale):
        if a == 0.0:
            np.testing.assert_array_equal(after[i], before[i])          # a frozen tensor does not move at all
    # refused: wrong values, mid-step
    with pytest.raises(B.GxpoError) as e:
        B.gxpo_set_tensor_options(ctx, [-1.0] * len(numels), wd_scale)
    assert e.value.code == B.GXPO_ERR_INVALID_ARG
    with pytest.raises(B.GxpoError) as e:
        B.gxpo_set_tensor_options(ctx, lr_scale, [float("nan")] * len(numels))
    assert e.value.code == B.GXPO_ERR_INVALID_ARG
    grad_fn(dev.views["theta"], grads[0])
    B.gxpo_fast_steps(ctx, 0, grads[0])
    with pytest.raises(B.GxpoError) as e:
        B.gxpo_set_tensor_options(ctx, lr_scale, wd_scale)
    assert e.value.code == B.GXPO_ERR_BAD_STATE


def test_unit_parameter_groups_change_nothing():
    """Multipliers of exactly 1 must leave every result bit-identical to a context that never set them."""
    numels = [4099, 257]
    problem = synth.policy_problem(sum(numels), seed=16, sigma=0.05, device="cuda")
    cfg = B.make_config(K=8, alpha=0.5, delta=1.75e-3, lr=1e-4, weight_decay=0.01, gate_min_count=2)
    runs = []
    for set_them in (False, True):
        dev, ctx, orc, grads = build(numels, cfg, problem)
        if set_them:
            B.gxpo_set_tensor_options(ctx, [1.0, 1.0], [1.0, 1.0])
        grad_fn = quad_trainer(problem, numels, step_noise=lambda: synth.step_noise(problem, 0))
        H.lockstep_active_step(ctx, dev, orc, grad_fn, grads, dtol=1e-4, fused=True, what="unit groups")
        runs.append([x.clone() for k in ("theta", "m", "v") for x in dev.views[k]])
    for a, b in zip(*runs):
        assert torch.equal(a, b)


@pytest.mark.parametrize("fused", [True, False])
def test_all_inactive_equals_lookahead_depth_two(fused):
    """delta = +inf switches every coordinate off the active set (scale = 1 everywhere); K = 2 makes the
    geometric factor 1 on the active set.  Both leave theta~ = theta + alpha (theta^{t,2} - theta): the two
    configurations must agree bit for bit, and with the oracle."""
    numels = [4099, 257, 70001]
    problem = synth.policy_problem(sum(numels), seed=17, sigma=0.05, device="cuda")
    results = []
    for kwargs in (dict(K=8, delta=math.inf), dict(K=2, delta=0.0), dict(K=9, delta=math.inf)):
        cfg = B.make_config(alpha=0.5, lr=1e-4, weight_decay=0.01, fuse_step2=fused, gate_min_count=2, **kwargs)
        dev, ctx, orc, grads = build(numels, cfg, problem)
        grad_fn = quad_trainer(problem, numels, step_noise=lambda: synth.step_noise(problem, 0))
        H.lockstep_active_step(ctx, dev, orc, grad_fn, grads, dtol=1e-4, fused=fused, what=f"{kwargs}")
        assert all(np.all(s == 1.0) for s in orc.scale)
        results.append([x.clone() for k in ("theta", "m", "v") for x in dev.views[k]])
    for other in results[1:]:
        for a, b in zip(results[0], other):
            assert torch.equal(a, b)


def test_checkpoint_and_resume_is_bit_identical():
    """Six steps in one go against three steps, a checkpoint (the caller's buffers plus gxpo_get_state),
    a brand-new context restored with gxpo_set_state, and three more steps: same bits, same gate records."""
    numels = [4099, 257, 70001]
    problem = synth.policy_problem(sum(numels), seed=18, sigma=0.05, device="cuda")
    cfg = B.make_config(K=8, alpha=0.5, delta=1.75e-3, lr=1e-4, weight_decay=0.01, gate_min_count=2, window=3, tau=1e6)
    step_id = [0]
    grad_fn = quad_trainer(problem, numels, step_noise=lambda: synth.step_noise(problem, step_id[0]))

    def run_steps(ctx, dev, grads, steps):
        infos = []
        for step in steps:
            step_id[0] = step
            g0, g1, gs = grads
            grad_fn(dev.views["theta"], g0); B.gxpo_fast_steps(ctx, 0, g0)
            grad_fn(dev.views["theta_probe"], g1); B.gxpo_fast_steps(ctx, 1, g1)
            B.gxpo_extrapolate(ctx, g0, g1)
            grad_fn(dev.views["theta"], gs); B.gxpo_slow_step(ctx, gs)
            i = B.gxpo_gate(ctx)
            infos.append((i.norm, i.mu, i.sigma, i.z, i.evaluated, i.t))
        return infos

    dev_a, ctx_a, _, grads_a = build(numels, cfg, problem)
    infos_a = run_steps(ctx_a, dev_a, grads_a, range(6))

    dev_b, ctx_b, _, grads_b = build(numels, cfg, problem)
    infos_b = run_steps(ctx_b, dev_b, grads_b, range(3))
    saved_state = B.gxpo_get_state(ctx_b)
    saved = {k: [x.clone() for x in dev_b.views[k]] for k in ("theta", "m", "v")}
    B.gxpo_destroy(ctx_b)
    del dev_b

    dev_c = H.DeviceState(numels, adam=True, with_copy=False)
    for k, xs in saved.items():
        for dst, src in zip(dev_c.views[k], xs):
            dst.copy_(src)
    ctx_c = B.gxpo_init(cfg, dev_c.tensor_dicts())
    B.gxpo_set_state(ctx_c, saved_state)
    infos_b += run_steps(ctx_c, dev_c, grads_b, range(3, 6))

    same = lambda a, b: all((x == y) or (x != x and y != y) for x, y in zip(a, b))       # NaN == NaN during warm-up
    assert all(same(a, b) for a, b in zip(infos_a, infos_b)) and len(infos_b) == 6
    for k in ("theta", "m", "v"):
        for a, c in zip(dev_a.views[k], dev_c.views[k]):
            assert torch.equal(a, c), f"{k} differs after resume"
    sa, sc = B.gxpo_get_state(ctx_a), B.gxpo_get_state(ctx_c)
    assert (sa.t, sa.optim_steps, sa.backward_passes, sa.window_len, list(sa.window[:3])) == \
           (sc.t, sc.optim_steps, sc.backward_passes, sc.window_len, list(sc.window[:3])) and sa.t == 6


def test_two_contexts_interleaved_on_two_streams_do_not_interact():
    """Contexts own their workspace: two of them, driven call by call on two side streams,
    give exactly what each gives alone."""
    specs = [([4099, 257], 19, dict(K=8, alpha=0.5, lr=1e-4)), ([70001], 20, dict(K=5, alpha=1.0, lr=3e-5, clip_norm=5.0, diagnostics=1))]

    def make(numels, seed, kw):
        problem = synth.policy_problem(sum(numels), seed=seed, sigma=0.05, device="cuda")
        cfg = B.make_config(delta=1.75e-3, weight_decay=0.01, gate_min_count=2, tau=1e6, **kw)
        dev, ctx, _, grads = build(numels, cfg, problem)
        return dict(problem=problem, numels=numels, dev=dev, ctx=ctx, grads=grads,
                    grad_fn=quad_trainer(problem, numels, step_noise=lambda: synth.step_noise(problem, 0)))

    def calls(r):
        g0, g1, gs = r["grads"]
        dev, ctx, grad_fn = r["dev"], r["ctx"], r["grad_fn"]
        yield lambda: (grad_fn(dev.views["theta"], g0), B.gxpo_fast_steps(ctx, 0, g0))
        yield lambda: (grad_fn(dev.views["theta_probe"], g1), B.gxpo_fast_steps(ctx, 1, g1))
        yield lambda: B.gxpo_extrapolate(ctx, g0, g1)
        yield lambda: (grad_fn(dev.views["theta"], gs), B.gxpo_slow_step(ctx, gs))
        yield lambda: r.__setitem__("norm", B.gxpo_gate(ctx).norm)

    solo = [make(*sp) for sp in specs]
    for r in solo:
        for _ in range(2):
            for c in calls(r):
                c()
    pair = [make(*sp) for sp in specs]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for _ in range(2):
        for ca, cb in zip(calls(pair[0]), calls(pair[1])):
            with torch.cuda.stream(streams[0]):
                ca()
            with torch.cuda.stream(streams[1]):
                cb()
    torch.cuda.synchronize()
    for a, b in zip(solo, pair):
        assert a["norm"] == b["norm"]
        for k in ("theta", "m", "v"):
            for x, y in zip(a["dev"].views[k], b["dev"].views[k]):
                assert torch.equal(x, y)


def test_fresh_gradient_buffers_on_every_call():
    """A trainer that hands in newly allocated gradient tensors on every call makes the engine re-validate and
    re-upload its pointer tables each time (more uploads than it has staging slots): same bits as with fixed buffers."""
    numels = [4099, 257, 1000]
    problem = synth.policy_problem(sum(numels), seed=24, sigma=0.05, device="cuda")
    cfg = B.make_config(K=8, alpha=0.5, delta=1.75e-3, lr=1e-4, weight_decay=0.01, gate_min_count=2, tau=1e6)
    grad_fn = quad_trainer(problem, numels, step_noise=lambda: synth.step_noise(problem, 0))
    outs = []
    for fresh in (False, True):
        dev, ctx, _, fixed = build(numels, cfg, problem)
        keep = []                                            # fresh buffers stay alive (and distinct) until the end
        for step in range(6):
            bufs = [H.grad_buffers(numels, torch.float32) for _ in range(3)] if fresh else fixed
            keep.append(bufs)
            g0, g1, gs = bufs
            grad_fn(dev.views["theta"], g0); B.gxpo_fast_steps(ctx, 0, g0)
            grad_fn(dev.views["theta_probe"], g1); B.gxpo_fast_steps(ctx, 1, g1)
            B.gxpo_extrapolate(ctx, g0, g1)
            grad_fn(dev.views["theta"], gs); B.gxpo_slow_step(ctx, gs)
            norm = B.gxpo_gate(ctx).norm
        outs.append((norm, [x.clone() for k in ("theta", "m", "v") for x in dev.views[k]]))
    assert outs[0][0] == outs[1][0]
    for a, b in zip(outs[0][1], outs[1][1]):
        assert torch.equal(a, b)


def test_hyper_parameter_schedule_through_update_config():
    """A learning-rate / alpha / K / delta schedule between steps: the engine with gxpo_update_config
    against the oracle whose configuration is changed the same way."""
    numels = [4099, 70001]
    problem = synth.policy_problem(sum(numels), seed=14, sigma=0.05, device="cuda")
    base = dict(delta=1.75e-3, weight_decay=0.01, gate_min_count=2, window=4, fuse_step2=True, tau=1e6)    # never trips
    schedule = [dict(lr=1e-4, alpha=0.5, K=5), dict(lr=5e-5, alpha=0.25, K=8), dict(lr=2e-5, alpha=1.0, K=3, delta=1e-2, gate_eps=1e-3),
                dict(lr=2e-5, alpha=0.5, K=4, r_max=2.0, window=2)]
    cfg = B.make_config(**base, **schedule[0])
    dev, ctx, orc, grads = build(numels, cfg, problem)
    step_id = [0]
    grad_fn = quad_trainer(problem, numels, step_noise=lambda: synth.step_noise(problem, step_id[0]))
    for step, hp in enumerate(schedule):
        step_id[0] = step
        if step:
            cfg = B.make_config(**{**base, **hp})
            B.gxpo_update_config(ctx, cfg)
            oc = H.oracle_config(cfg)
            orc.cfg, orc.gate.cfg = oc, oc.gate
            if len(orc.gate.buffer) > oc.gate.window:
                del orc.gate.buffer[:len(orc.gate.buffer) - oc.gate.window]
        H.lockstep_active_step(ctx, dev, orc, grad_fn, grads, dtol=1e-4, fused=True, what=f"schedule step {step}")
    st = B.gxpo_get_state(ctx)
    assert st.window_len == 2 and list(st.window[:2]) == orc.gate.buffer
    # what shapes the workspace cannot change; nothing changes in the middle of a step
    for bad in (dict(optimizer="gd"), dict(grad_dtype="bf16"), dict(fuse_step2=False),
                dict(diagnostics=1), dict(explicit_steps=3), dict(clip_norm=1.0)):
        with pytest.raises(B.GxpoError) as e:
            B.gxpo_update_config(ctx, B.make_config(**{**base, **schedule[0], **bad}))
        assert e.value.code == B.GXPO_ERR_INVALID_ARG, bad
    with pytest.raises(B.GxpoError) as e:
        B.gxpo_update_config(ctx, B.make_config(**{**base, **schedule[0], "K": 1}))
    assert e.value.code == B.GXPO_ERR_INVALID_ARG
    grad_fn(dev.views["theta"], grads[0])
    B.gxpo_fast_steps(ctx, 0, grads[0])
    with pytest.raises(B.GxpoError) as e:
        B.gxpo_update_config(ctx, cfg)
    assert e.value.code == B.GXPO_ERR_BAD_STATE


def test_non_finite_slow_gradient_trips_the_gate():
    """A NaN or infinite ||g_slow|| can never satisfy Z >= tau by comparison; the engine trips on it."""
    n = 5000
    for poison in (float("nan"), float("inf")):
        problem = synth.policy_problem(n, seed=4, device="cuda")
        dev, ctx, orc, grads = build([n], B.make_config(gate_min_count=2, lr=1e-4), problem)
        g0, g1, gs = grads
        for buf in (g0[0], g1[0], gs[0]):
            buf.copy_(torch.randn(n, device="cuda"))
        B.gxpo_fast_steps(ctx, 0, g0); B.gxpo_fast_steps(ctx, 1, g1); B.gxpo_extrapolate(ctx, g0, g1)
        gs[0][n // 2] = poison
        B.gxpo_slow_step(ctx, gs)
        info = B.gxpo_gate(ctx)
        ref = O.RollingGate(H.oracle_config(ctx.cfg).gate).step(0, float(info.norm))
        assert not math.isfinite(info.norm) and info.tripped and not info.evaluated and info.s_star == 1 == ref.s_star
        with pytest.raises(B.GxpoError):
            B.gxpo_fast_steps(ctx, 0, g0)                  # fallback phase from t = 1 on


@pytest.mark.parametrize("mode", ["fused", "unfused", "explicit"])
def test_random_call_sequences_follow_the_state_machine(mode):
    """600 randomly chosen calls per mode against a few-line model of Algorithm 1's call order: every call the
    model allows must succeed, every other one must be refused with BAD_STATE and change nothing."""
    n = 300
    n_fast = 3 if mode == "explicit" else 2
    cfg = B.make_config(fuse_step2=(mode == "fused"), explicit_steps=(3 if mode == "explicit" else 0), lr=1e-4, gate_min_count=2,
                        window=4, tau=1e6)
    problem = synth.policy_problem(n, seed=25, device="cuda")
    dev, ctx, _, _ = build([n], cfg, problem)
    g = [[torch.randn(n, device="cuda")] for _ in range(4)]
    rng = np.random.default_rng({"fused": 1, "unfused": 2, "explicit": 3}[mode])
    phase, fast_done, t, s_star, optim_steps, passes = "idle", 0, 0, None, 0, 0
    n_ok = 0
    for _ in range(600):
        fallback = s_star is not None and t >= s_star
        op = rng.choice(["fast", "extrapolate", "slow", "gate", "fallback", "trip", "rearm"], p=[0.3, 0.2, 0.2, 0.2, 0.05, 0.025, 0.025])
        which = int(rng.integers(0, n_fast))
        if rng.random() < 0.5:                  # half of the time, the call Algorithm 1 would make next
            op = {"idle": "fallback" if fallback else "fast", "fast": "fast", "fast_done": "extrapolate",
                  "repositioned": "slow", "slow_done": "gate"}[phase]
            which = fast_done if phase == "fast" else 0
        if op == "fast":
            legal = not fallback and ((which == 0 and phase == "idle") or (which > 0 and phase == "fast" and fast_done == which))
            call = lambda: B.gxpo_fast_steps(ctx, which, g[min(which, 1)])
        elif op == "extrapolate":
            legal = phase == "fast_done"
            call = (lambda: B.gxpo_extrapolate(ctx)) if mode == "explicit" else (lambda: B.gxpo_extrapolate(ctx, g[0], g[1]))
        elif op == "slow":
            legal = phase == "repositioned"
            call = lambda: B.gxpo_slow_step(ctx, g[2])
        elif op == "gate":
            legal = phase == "slow_done"
            call = lambda: B.gxpo_gate(ctx)
        elif op == "fallback":
            legal = fallback and phase == "idle"
            call = lambda: B.gxpo_fallback_step(ctx, g[3])
        else:                                   # flip the gate through the state interface (legal between steps only)
            legal = phase == "idle"
            new_star = t if op == "trip" else -1

            def call(new_star=new_star):
                st = B.gxpo_get_state(ctx)
                st.s_star = new_star
                B.gxpo_set_state(ctx, st)
        if legal:
            call()
            n_ok += 1
            if op == "fast":
                fast_done, optim_steps, passes = which + 1, optim_steps + 1, passes + 1
                phase = "fast_done" if fast_done == n_fast else "fast"
            elif op == "extrapolate":
                phase = "repositioned"
            elif op == "slow":
                phase, optim_steps, passes = "slow_done", optim_steps + 1, passes + 1
            elif op == "gate":
                phase, t = "idle", t + 1
            elif op == "fallback":
                t, optim_steps, passes = t + 1, optim_steps + 1, passes + 1
            elif op == "trip":
                s_star = t
            else:
                s_star = None
        else:
            with pytest.raises(B.GxpoError) as e:
                call()
            assert e.value.code == B.GXPO_ERR_BAD_STATE, (op, which, phase, e.value.message)
        st = B.gxpo_get_state(ctx)
        assert (st.t, st.optim_steps, st.backward_passes, st.s_star) == (t, optim_steps, passes, -1 if s_star is None else s_star)
    assert n_ok > 100
    torch.cuda.synchronize()
    dev.check_canaries()


def test_init_rejects_host_memory_and_short_allocations():
    n = 4096
    cfg = B.make_config(optimizer="gd")
    theta = torch.zeros(n, device="cuda")
    probe = torch.zeros(n, device="cuda")
    arr = (B.gxpo_tensor * 1)()
    arr[0].numel = 1 << 24                              # far beyond the 16 KiB allocation
    arr[0].theta, arr[0].theta_probe = theta.data_ptr(), probe.data_ptr()
    import ctypes
    out = ctypes.c_void_p()
    assert B._lib.gxpo_init(ctypes.byref(out), ctypes.byref(cfg), arr, 1) == B.GXPO_ERR_INVALID_ARG
    host = torch.zeros(n)
    arr[0].numel = n
    arr[0].theta = host.data_ptr()
    assert B._lib.gxpo_init(ctypes.byref(out), ctypes.byref(cfg), arr, 1) == B.GXPO_ERR_INVALID_ARG
    assert out.value is None


# ---------------------------------------------------------------------------------------------
# reduction: reproducible, per-tensor, many blocks
# ---------------------------------------------------------------------------------------------
def test_norm_reduction_is_bit_reproducible_and_matches_oracle():
    numels = [3 * 8192 * 256 + 11, 5, 700001]           # first tensor spans more than one reduction run
    cfg = B.make_config(optimizer="gd", lr=1e-3, gate_min_count=2)
    results = []
    g = H.grad_buffers(numels, torch.float32)
    gen = torch.Generator(device="cuda").manual_seed(5)
    for x in g:
        x.copy_(torch.randn(x.numel(), generator=gen, device="cuda") * 0.05)
    for rep in range(2):
        dev = H.DeviceState(numels, adam=False, with_copy=False)
        for x in dev.views["theta"]:
            x.zero_()
        ctx = B.gxpo_init(cfg, dev.tensor_dicts())
        g1 = [x.clone() for x in g]
        B.gxpo_fast_steps(ctx, 0, g); B.gxpo_fast_steps(ctx, 1, g1); B.gxpo_extrapolate(ctx, g, g1); B.gxpo_slow_step(ctx, g)
        info = B.gxpo_gate(ctx)
        results.append((info.norm, tuple(B.gxpo_tensor_norms(ctx))))
        B.gxpo_destroy(ctx)
    assert results[0] == results[1]                      # bit-identical from run to run
    want = [math.sqrt(O.sum_squares(H.f64(x))) for x in g]
    for a, b in zip(results[0][1], want):
        assert a == pytest.approx(b, rel=1e-13)
    assert results[0][0] == pytest.approx(math.sqrt(sum(w * w for w in want)), rel=1e-13)


def test_plain_c_program_drives_the_library():
    """No Python, no torch in the process: a gcc-built C99 program allocates with the HIP runtime's C API,
    calls the engine through include/gxpo.h and checks the paper's closed form for the diagonal surrogate."""
    import os
    import subprocess
    from paper_2605_06755_amd import build as lib_build
    if not os.path.exists(lib_build.ABI_DRIVER):
        pytest.fail(f"{lib_build.ABI_DRIVER} is not built: run __graft_entry__.build() first")
    res = subprocess.run([lib_build.ABI_DRIVER], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert res.returncode == 0 and res.stdout.strip().endswith("abi driver ok"), res.stdout


def test_stream_copy_reference_kernel():
    for n in (4, 256, 260, 1 << 20, (1 << 20) + 12):
        src = torch.randn(n, device="cuda")
        dst = torch.full((n + 8,), 7.0, device="cuda")
        B.gxpo_stream_copy(dst[:n], src)
        torch.cuda.synchronize()
        assert torch.equal(dst[:n], src) and bool((dst[n:] == 7.0).all())


# ---------------------------------------------------------------------------------------------
# the fused schedule's replay: theta^{t,1}, m, v bit for bit what the unfused passes store
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("optimizer", ["adamw", "gd"])
@pytest.mark.parametrize("grad_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("clip_norm", [0.0, 5.0])
def test_fused_replay_is_bit_identical_to_the_unfused_passes(optimizer, grad_dtype, clip_norm):
    """Same inputs through fuse_step2 = 1 and = 0, three steps.  What the header promises bit for bit:
    theta^{t,1} as the probe pass previews it equals what the unfused first fast step stores, and m, v after
    gxpo_extrapolate (fused: both moment updates applied in the replay) equal m, v after the unfused second
    fast step.  theta~ is NOT promised bit-equal: the unfused path rounds theta^{t,2} to fp32 before the
    displacement is formed, the fused pass forms (theta^{t,1} - theta^t) - update_2 without that rounding;
    the two may differ by that one rounding times alpha * scale, which is what is asserted."""
    numels = RAGGED
    P = sum(numels)
    problem = synth.policy_problem(P, seed=31, sigma=0.05, device="cuda")
    common = dict(optimizer=optimizer, grad_dtype=grad_dtype, K=5, alpha=0.5, delta=1.75e-3, lr=1e-3 if optimizer == "gd" else 1e-4,
                  weight_decay=0.01, gate_min_count=2, clip_norm=clip_norm, copy_mask=7, r_max=4.0)
    runs = {}
    for fused in (True, False):
        cfg = B.make_config(fuse_step2=fused, **common)
        dev, ctx, orc, grads = build(numels, cfg, problem, with_copy=True)
        runs[fused] = (dev, ctx, orc, grads)
    grad_fn = quad_trainer(problem, numels, step_noise=lambda: synth.step_noise(problem, step_id[0]))
    step_id = [0]
    adam = optimizer == "adamw"
    bits = lambda dev, key: [x.clone() for x in dev.views[key]]
    raw = lambda x: x.view(torch.int32) if x.element_size() == 4 else x.view(torch.int16)
    same = lambda a, b: all(torch.equal(raw(x), raw(y)) for x, y in zip(a, b))
    for step in range(3):
        step_id[0] = step
        snap = {}
        for k in runs[False][0].views:                       # both schedules start every step from the same state
            for dst, src in zip(runs[False][0].views[k], runs[True][0].views[k]):
                dst.copy_(src)
        for fused in (True, False):
            dev, ctx, orc, (g0b, g1b, gsb) = runs[fused]
            st = B.gxpo_get_state(ctx)
            H.sync_oracle_to_device(orc, dev, st.optim_steps)
            grad_fn(dev.views["theta"], g0b)
            B.gxpo_fast_steps(ctx, 0, g0b)
            snap[fused, "th1"] = bits(dev, "theta_probe")
            snap[fused, "copy1"] = bits(dev, "model_copy")
            orc.fast_step_1([H.f64(g) for g in g0b])
            grad_fn(dev.views["theta_probe"], g1b)
            B.gxpo_fast_steps(ctx, 1, g1b)
            orc.fast_step_2([H.f64(g) for g in g1b])
            snap[fused, "theta_before"] = bits(dev, "theta")
            B.gxpo_extrapolate(ctx, g0b, g1b)
            orc.extrapolate([H.f64(g) for g in g0b], [H.f64(g) for g in g1b])
            snap[fused, "tilde"] = bits(dev, "theta")
            if adam:
                snap[fused, "m"], snap[fused, "v"] = bits(dev, "m"), bits(dev, "v")
            snap[fused, "scale"] = [s.copy() for s in orc.scale]
            snap[fused, "th2"] = [t.copy() for t in orc._theta_2]
            snap[fused, "g"] = [g.clone() for g in g0b + g1b]
        # identical inputs went in
        assert same(snap[True, "g"], snap[False, "g"]) and same(snap[True, "theta_before"], snap[False, "theta_before"])
        # the promise
        assert same(snap[True, "th1"], snap[False, "th1"]), f"step {step}: previewed theta^(t,1) differs from the stored one"
        assert all(torch.equal(a.view(torch.int16), b.view(torch.int16)) for a, b in zip(snap[True, "copy1"], snap[False, "copy1"]))
        if adam:
            assert same(snap[True, "m"], snap[False, "m"]), f"step {step}: m after the replay differs"
            assert same(snap[True, "v"], snap[False, "v"]), f"step {step}: v after the replay differs"
        # theta~: one fp32 rounding of theta^{t,2}, multiplied by alpha * scale
        for a, b, sc, th0, th2 in zip(snap[True, "tilde"], snap[False, "tilde"], snap[True, "scale"], snap[True, "theta_before"],
                                      snap[True, "th2"]):
            a64, b64 = H.f64(a), H.f64(b)
            mag = np.maximum(np.maximum(np.abs(b64), np.abs(H.f64(th0))), np.abs(th2))      # the iterates' magnitude sets the ulp
            bound = 2.0 ** -23 * mag * (1.0 + common["alpha"] * np.abs(sc))
            assert np.all(np.abs(a64 - b64) <= bound), f"step {step}: theta~ differs by more than the rounding of theta^(t,2)"
        # finish the step on both (slow step from each schedule's own theta~)
        for fused in (True, False):
            dev, ctx, orc, (g0b, g1b, gsb) = runs[fused]
            grad_fn(dev.views["theta"], gsb)
            B.gxpo_slow_step(ctx, gsb)
            B.gxpo_gate(ctx)
    for fused in (True, False):
        B.gxpo_destroy(runs[fused][1])


@pytest.mark.gpu
@pytest.mark.parametrize("grad_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("clip_norm,diagnostics", [(0.0, False), (0.5, False), (0.0, True)])
def test_alternating_state_is_bit_identical_to_the_in_place_schedule(grad_dtype, clip_norm, diagnostics):
    """Two buffer sets ({theta, m, v} and {theta_probe, m_alt, v_alt}): every state-advancing pass reads one and
    writes the other.  Same inputs through the in-place schedule (checked against the oracle by the other tests)
    and the alternating one: after every call the iterate the call produces, the moments, the bf16 copy, the
    norm and the gate's decision are bit-identical, they are where gxpo_state.current_set says, and the set
    that was read is untouched.  Active steps, then fallback steps (which alternate), then a resume from a
    checkpoint taken while set 1 was current.  (The alternating schedule is also compared with the oracle
    directly, call by call, in test_adamw_ragged_lockstep.)"""
    numels = RAGGED
    P = sum(numels)
    problem = synth.policy_problem(P, seed=41, sigma=0.05, device="cuda")
    cfg = B.make_config(optimizer="adamw", grad_dtype=grad_dtype, K=6, alpha=0.5, delta=1.75e-3, lr=1e-4, weight_decay=0.01,
                        clip_norm=clip_norm, diagnostics=diagnostics, copy_mask=7, r_max=4.0, tau=1e9)
    ref_dev, ref_ctx, orc, (g0, g1, gs) = build(numels, cfg, problem, with_copy=True)
    alt_dev, alt_ctx, _, _ = build(numels, cfg, problem, with_copy=True, alternating=True)
    step_id = [0]
    grad_fn = quad_trainer(problem, numels, step_noise=lambda: synth.step_noise(problem, step_id[0]))
    raw = lambda x: x.view(torch.int32) if x.element_size() == 4 else x.view(torch.int16)

    def same(key_ref, key_alt, what):
        for i, (a, b) in enumerate(zip(ref_dev.views[key_ref], alt_dev.views[key_alt])):
            assert torch.equal(raw(a), raw(b)), f"{what}: tensor {i}, {key_ref} (in place) differs from {key_alt} (alternating)"

    def same_state(what):
        cur = B.gxpo_get_state(alt_ctx).current_set
        th, m, v = H.DeviceState.set_keys(cur)
        assert [x.data_ptr() for x in B.gxpo_current_params(alt_ctx)] == [x.data_ptr() for x in alt_dev.views[th]]
        assert [x.data_ptr() for x in B.gxpo_current_params(ref_ctx)] == [x.data_ptr() for x in ref_dev.views["theta"]]
        same("theta", th, what), same("m", m, what), same("v", v, what), same("model_copy", "model_copy", what)
        return cur

    def snapshot(cur):
        return [x.clone() for k in H.DeviceState.set_keys(cur) for x in alt_dev.views[k]]

    def untouched(cur, before, what):
        now = [x for k in H.DeviceState.set_keys(cur) for x in alt_dev.views[k]]
        assert all(torch.equal(raw(a), raw(b)) for a, b in zip(before, now)), f"{what}: the set that was read has changed"

    def both(fn):
        return fn(ref_ctx), fn(alt_ctx)

    assert B.gxpo_get_state(alt_ctx).current_set == 0 and B.gxpo_get_state(ref_ctx).current_set == 0
    for step in range(3):
        step_id[0] = step
        c = B.gxpo_get_state(alt_ctx).current_set
        assert c == 0                                               # an active step ends in the set it started in
        th_c, _, _ = H.DeviceState.set_keys(c)
        th_o, _, _ = H.DeviceState.set_keys(1 - c)
        grad_fn(ref_dev.views["theta"], g0)
        before = snapshot(c)
        both(lambda ctx: B.gxpo_fast_steps(ctx, 0, g0))
        same("theta_probe", th_o, f"step {step}, theta^(t,1)")
        untouched(c, before, f"step {step}, first fast step")
        grad_fn(ref_dev.views["theta_probe"], g1)
        both(lambda ctx: B.gxpo_fast_steps(ctx, 1, g1))
        both(lambda ctx: B.gxpo_extrapolate(ctx, g0, g1))
        assert B.gxpo_get_state(alt_ctx).current_set == 1 - c and B.gxpo_get_state(ref_ctx).current_set == 0
        same_state(f"step {step}, after gxpo_extrapolate")
        untouched(c, before, f"step {step}, gxpo_extrapolate")      # theta^t, m, v of the step's start are still there
        grad_fn(ref_dev.views["theta"], gs)
        before = snapshot(1 - c)
        both(lambda ctx: B.gxpo_slow_step(ctx, gs))
        assert B.gxpo_get_state(alt_ctx).current_set == c
        same_state(f"step {step}, after gxpo_slow_step")
        untouched(1 - c, before, f"step {step}, gxpo_slow_step")
        assert B.gxpo_tensor_norms(ref_ctx) == B.gxpo_tensor_norms(alt_ctx)
        if diagnostics:
            da, db = both(B.gxpo_get_diagnostics)
            assert all(getattr(da, k) == getattr(db, k) or (getattr(da, k) != getattr(da, k) and getattr(db, k) != getattr(db, k))
                       for k, _ in da._fields_)
        ia, ib = both(B.gxpo_gate)
        assert (ia.norm, ia.tripped, ia.s_star) == (ib.norm, ib.tripped, ib.s_star)
    alt_dev.check_canaries()

    # fallback steps alternate between the sets
    for ctx in (ref_ctx, alt_ctx):
        st = B.gxpo_get_state(ctx)
        st.s_star = st.t
        B.gxpo_set_state(ctx, st)
    checkpoint = None
    for k in range(3):
        step_id[0] = 10 + k
        c = B.gxpo_get_state(alt_ctx).current_set
        assert c == k % 2
        grad_fn(ref_dev.views["theta"], g0)
        before = snapshot(c)
        both(lambda ctx: B.gxpo_fallback_step(ctx, g0))
        assert same_state(f"fallback step {k}") == 1 - c
        untouched(c, before, f"fallback step {k}")
        if k == 0:
            checkpoint = B.gxpo_get_state(alt_ctx)                  # set 1 is current here
            saved = {key: [x.clone() for x in alt_dev.views[key]] for key in alt_dev.views}
    assert checkpoint.current_set == 1
    final = {key: [x.clone() for x in alt_dev.views[key]] for key in ("theta", "theta_probe", "m", "v", "m_alt", "v_alt", "model_copy")}

    # resume from the checkpoint in a new context: the same two fallback steps give the same bits
    B.gxpo_destroy(alt_ctx)
    for key, views in saved.items():
        for dst, src in zip(alt_dev.views[key], views):
            dst.copy_(src)
    alt_ctx = B.gxpo_init(cfg, alt_dev.tensor_dicts())
    B.gxpo_set_state(alt_ctx, checkpoint)
    for k in (1, 2):
        step_id[0] = 10 + k
        cur = H.DeviceState.set_keys(B.gxpo_get_state(alt_ctx).current_set)[0]
        grad_fn(alt_dev.views[cur], g0)
        B.gxpo_fallback_step(alt_ctx, g0)
    for key, views in final.items():
        if key in H.DeviceState.set_keys(B.gxpo_get_state(alt_ctx).current_set) or key == "model_copy":
            assert all(torch.equal(raw(a), raw(b)) for a, b in zip(views, alt_dev.views[key])), f"resume: {key} differs"
    alt_dev.check_canaries()

    # an in-place context has no second set to point at
    st = B.gxpo_get_state(ref_ctx)
    st.current_set = 1
    with pytest.raises(B.GxpoError) as e:
        B.gxpo_set_state(ref_ctx, st)
    assert e.value.code == B.GXPO_ERR_INVALID_ARG
    B.gxpo_destroy(ref_ctx)
    B.gxpo_destroy(alt_ctx)


@pytest.mark.gpu
def test_alternating_state_is_refused_where_it_cannot_work():
    numels = [1000, 4099]
    dev = H.DeviceState(numels, True, False, alternating=True)
    ok = B.make_config(optimizer="adamw")
    for bad in (dict(fuse_step2=False), dict(explicit_steps=3)):
        with pytest.raises(B.GxpoError) as e:
            B.gxpo_init(B.make_config(optimizer="adamw", **bad), dev.tensor_dicts())
        assert e.value.code == B.GXPO_ERR_UNSUPPORTED
    dicts = dev.tensor_dicts()
    del dicts[1]["v_alt"]                                           # half a pair
    with pytest.raises(B.GxpoError) as e:
        B.gxpo_init(ok, dicts)
    assert e.value.code == B.GXPO_ERR_INVALID_ARG
    dicts = dev.tensor_dicts()
    del dicts[1]["m_alt"], dicts[1]["v_alt"]                        # one tensor with, one without
    with pytest.raises(B.GxpoError) as e:
        B.gxpo_init(ok, dicts)
    assert e.value.code == B.GXPO_ERR_INVALID_ARG
    dicts = dev.tensor_dicts()
    for d in dicts:
        del d["theta_probe"]                                        # no second parameter buffer
    with pytest.raises(B.GxpoError) as e:
        B.gxpo_init(ok, dicts)
    assert e.value.code == B.GXPO_ERR_INVALID_ARG
    dicts = dev.tensor_dicts()
    dicts[0]["m_alt"] = dicts[0]["m"]                               # aliasing the first set
    with pytest.raises(B.GxpoError) as e:
        B.gxpo_init(ok, dicts)
    assert e.value.code == B.GXPO_ERR_INVALID_ARG
    ctx = B.gxpo_init(ok, dev.tensor_dicts())                       # and the plain case works
    B.gxpo_destroy(ctx)


# ---------------------------------------------------------------------------------------------
# a NULL entry in a gradient list is refused on the host, whatever has been staged before
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("n_tensors", [1, 3])
def test_null_gradient_entry_is_refused_before_any_launch(fused, n_tensors):
    import ctypes
    numels = [4099, 1000, 257][:n_tensors]
    problem = synth.policy_problem(sum(numels), seed=41, sigma=0.05, device="cuda")
    cfg = B.make_config(K=5, alpha=0.5, delta=1.75e-3, lr=1e-4, fuse_step2=fused, gate_min_count=2)
    dev, ctx, orc, (g0b, g1b, gsb) = build(numels, cfg, problem)
    for g in g0b + g1b + gsb:
        g.normal_(std=0.05)
    stream = B._stream_ptr(None)

    def ptrs(bufs, null_at=None):
        return (ctypes.c_void_p * n_tensors)(*[None if i == null_at else b.data_ptr() for i, b in enumerate(bufs)])

    def state_bits():
        torch.cuda.synchronize()
        return {k: torch.cat([x.view(torch.int32).reshape(-1) for x in v]).clone() for k, v in dev.views.items()}

    def refused(call, label):
        before, phase = state_bits(), B.gxpo_get_state(ctx).phase
        rc = call()
        assert rc == B.GXPO_ERR_INVALID_ARG, f"{label}: rc {rc}"
        assert "NULL" in B.gxpo_last_error(ctx) or "differs" in B.gxpo_last_error(ctx), B.gxpo_last_error(ctx)
        after = state_bits()
        assert B.gxpo_get_state(ctx).phase == phase, f"{label}: the state machine moved"
        assert all(torch.equal(before[k], after[k]) for k in before), f"{label}: a buffer was written"

    last = n_tensors - 1
    # first use of every role, with nothing staged yet
    refused(lambda: B._lib.gxpo_fast_steps(ctx.handle, 0, ptrs(g0b, null_at=last), stream), "g0, first use")
    B.gxpo_fast_steps(ctx, 0, g0b)
    refused(lambda: B._lib.gxpo_fast_steps(ctx.handle, 1, ptrs(g1b, null_at=0), stream), "g1, first use")
    B.gxpo_fast_steps(ctx, 1, g1b)
    refused(lambda: B._lib.gxpo_extrapolate(ctx.handle, ptrs(g0b, null_at=last), ptrs(g1b), stream), "extrapolate g0")
    refused(lambda: B._lib.gxpo_extrapolate(ctx.handle, ptrs(g0b), ptrs(g1b, null_at=0), stream), "extrapolate g1")
    B.gxpo_extrapolate(ctx, g0b, g1b)
    refused(lambda: B._lib.gxpo_slow_step(ctx.handle, ptrs(gsb, null_at=last), stream), "g_slow, first use")
    B.gxpo_slow_step(ctx, gsb)
    B.gxpo_gate(ctx)
    # and again once every role has valid pointers staged
    refused(lambda: B._lib.gxpo_fast_steps(ctx.handle, 0, ptrs(g0b, null_at=0), stream), "g0, second step")
    B.gxpo_destroy(ctx)
    # the fallback step's gradient on a context that has staged nothing
    dev, ctx, orc, (g0b, g1b, gsb) = build(numels, cfg, problem)
    st = B.gxpo_get_state(ctx)
    st.s_star = 0
    B.gxpo_set_state(ctx, st)
    refused(lambda: B._lib.gxpo_fallback_step(ctx.handle, ptrs(g0b, null_at=last), stream), "fallback, first use")
    B.gxpo_fallback_step(ctx, g0b)
    torch.cuda.synchronize()
    B.gxpo_destroy(ctx)
