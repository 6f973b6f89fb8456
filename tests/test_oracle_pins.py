"""Pins for the fp64 oracle: what the paper and the mathematics fix.

None of these tests re-types the oracle's formula.  Each compares the oracle
with something independent: an explicit K-step gradient-descent unroll, a
closed form, a library optimizer, numpy statistics, a bound the paper proves,
or a value the paper prints (tests/golden/, cited there).
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import gxpo_oracle as O
from paper_2605_06755_amd import synth


# ---------------------------------------------------------------------------
# helpers that are NOT the oracle: brute-force gradient descent, bounds
# ---------------------------------------------------------------------------
def gd_unroll(theta, grad_fn, eta, n_steps):
    th = theta.copy()
    for _ in range(n_steps):
        th = th - eta * grad_fn(th)
    return th


def surrogate_numpy(numel=1 << 14, seed=0):
    p = synth.surrogate_problem(numel, seed)
    return (p.h.double().numpy(), p.theta_star.double().numpy(), p.theta_0.double().numpy())


def gd_config(K, alpha, eta=0.1, delta=0.0):
    return O.GXPOConfig(optim=O.OptimConfig("gd", lr=eta), K=K, alpha=alpha, delta=delta,
                        gate=O.GateConfig(tau=3.0, window=10))


# ---------------------------------------------------------------------------
# 1. Diagonal quadratic + plain GD: the extrapolated point IS K explicit GD
#    steps, and a whole alpha = 1 outer step is K + 1 GD steps
#    (Section 2.4 corollary; Appendix A.6).
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("K", [2, 3, 4, 5, 8, 10])
def test_extrapolated_point_equals_K_gd_steps(K):
    h, ts, th0 = surrogate_numpy()
    eta = 0.1
    grad = lambda th: h * (th - ts)
    orc = O.GXPOOracle(gd_config(K, 1.0, eta), [th0])
    for step in range(5):
        start = orc.theta[0].copy()
        info = orc.train_step(lambda ths: [grad(ths[0])])
        want_K = gd_unroll(start, grad, eta, K)
        want_next = gd_unroll(start, grad, eta, K + 1)
        np.testing.assert_allclose(orc.theta_K[0], want_K, rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(orc.theta_tilde[0], want_K, rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(orc.theta[0], want_next, rtol=1e-11, atol=1e-13)
        assert not info.tripped
    assert orc.backward_passes == 15 and orc.optim_steps == 15


def test_config1_twenty_active_steps_closed_form():
    """P = 2^20, eta = 0.1, K = 4, alpha = 1, 20 active steps: theta_20 must be
    the 100th GD iterate, theta* + (1 - eta h)^100 (theta_0 - theta*)."""
    h, ts, th0 = surrogate_numpy(1 << 20, 0)
    eta, K = 0.1, 4
    orc = O.GXPOOracle(gd_config(K, 1.0, eta), [th0])
    norms = []
    for _ in range(20):
        info = orc.train_step(lambda ths: [h * (ths[0] - ts)])
        norms.append(info.norm)
        assert not info.tripped
    want = ts + (1.0 - eta * h) ** 100 * (th0 - ts)
    np.testing.assert_allclose(orc.theta[0], want, rtol=1e-10, atol=1e-12)
    assert all(b < a for a, b in zip(norms, norms[1:]))      # gradient norm only shrinks
    assert orc.s_star is None and orc.backward_passes == 60


@pytest.mark.parametrize("alpha", [0.0, 0.1, 0.5])
def test_partial_reposition_closed_form(alpha):
    """alpha < 1 on the diagonal quadratic: per outer step the error shrinks by
    rho (1 - alpha + alpha rho^K), rho = 1 - eta h (from Eq. (9) applied to the
    exact K-step point, then one GD step)."""
    h, ts, th0 = surrogate_numpy()
    eta, K, steps = 0.1, 4, 6
    orc = O.GXPOOracle(gd_config(K, alpha, eta), [th0])
    for _ in range(steps):
        orc.train_step(lambda ths: [h * (ths[0] - ts)])
    rho = 1.0 - eta * h
    want = ts + (rho * (1 - alpha + alpha * rho ** K)) ** steps * (th0 - ts)
    np.testing.assert_allclose(orc.theta[0], want, rtol=1e-11, atol=1e-13)


def test_loss_contraction_bound():
    """L(theta_m) <= rho^{(K+1) m} L(theta_0), rho = (1 - eta mu)^2, for the
    paper's L = 1/2 theta^T H theta with eta h_i <= 1 (Appendix A.6)."""
    h, _, th0 = surrogate_numpy()
    eta, K = 0.9, 5                       # eta * max h <= 0.9
    loss = lambda th: 0.5 * np.sum(h * th * th)
    orc = O.GXPOOracle(gd_config(K, 1.0, eta), [th0])
    rho = (1 - eta * h.min()) ** 2
    L0 = loss(th0)
    for m in range(1, 6):
        orc.train_step(lambda ths: [h * ths[0]])
        assert loss(orc.theta[0]) <= rho ** ((K + 1) * m) * L0 * (1 + 1e-9)


# ---------------------------------------------------------------------------
# 2. Special values of the extrapolation factor (Eq. (7); definition of S_K
#    in Appendix A.4; Algorithm 1's inactive branch)
# ---------------------------------------------------------------------------
def test_scale_special_values():
    for K in (2, 3, 4, 5, 8, 10):
        assert O.scale_factor(1.0, 1.0, K, 0.0) == K / 2            # r = 1  -> S_K/S_2 = K/2
        assert O.scale_factor(1.0, 0.0, K, 0.0) == 1.0              # r = 0  -> 1
        assert O.scale_factor(3.0, 7.0, K, math.inf) == 1.0         # delta = inf -> inactive
    for r in (-3.0, -0.5, 0.25, 0.9, 1.5, 2.0):
        assert O.scale_factor(2.0, 2.0 * r, 2, 0.0) == pytest.approx(1.0, rel=1e-15)   # K = 2
        for K in (3, 4, 5, 8, 10):
            closed = (1 - r ** K) / (1 - r ** 2)                    # Eq. (7), simplified form
            assert O.scale_factor(2.0, 2.0 * r, K, 0.0) == pytest.approx(closed, rel=1e-13)


def test_scale_uses_g1_over_g0_not_the_inverse():
    # r = 0.5: S_3/S_2 = 1.75/1.5; the inverse ratio r = 2 would give 7/3
    assert O.scale_factor(4.0, 2.0, 3, 0.0) == pytest.approx(1.75 / 1.5, rel=1e-15)


def test_geometric_sum_is_the_sum():
    for x in (-2.0, -1.0, -0.3, 0.0, 0.7, 1.0, 1.0 + 1e-9, 3.0):
        for n in (1, 2, 3, 7, 10):
            assert O.geometric_sum(x, n) == pytest.approx(sum(x ** j for j in range(n)), rel=1e-14)
    assert O.geometric_sum(1.0, 8) == 8.0


def test_active_set_is_strict_and_uses_abs():
    d = 0.5                                               # exactly representable in fp32
    assert O.scale_factor(0.5, 0.5, 4, d) == 1.0          # |g0| == delta -> inactive
    assert O.scale_factor(-0.5, -0.5, 4, d) == 1.0
    assert O.scale_factor(np.nextafter(np.float32(0.5), np.float32(1)), 0.5, 4, d) != 1.0
    assert O.scale_factor(-0.75, -0.75, 4, d) == 2.0      # negative g0 is active by magnitude
    assert O.scale_factor(0.0, 1.0, 4, 0.0) == 1.0        # g0 = 0 never forms a ratio


def test_delta_threshold_is_taken_in_fp32():
    d = 1e-8                                              # not an fp32 number
    d32 = float(np.float32(d))
    lo, hi = sorted((d, d32))
    mid = 0.5 * (lo + hi)                                 # between delta and fp32(delta)
    expect_active = mid > d32
    assert (O.scale_factor(mid, mid, 4, d) == 2.0) == expect_active


def test_inactive_and_alpha_edges_in_extrapolate():
    rng = np.random.default_rng(1)
    n = 257
    th0, th2 = rng.normal(size=n), rng.normal(size=n)
    g0, g1 = rng.normal(size=n), rng.normal(size=n)
    g0[::5] = 0.0
    # alpha = 0 ignores the prediction; alpha = 1 adopts it
    s, tk, tt = O.extrapolate(th0, th2, g0, g1, 5, 0.0, 1e-3)
    np.testing.assert_array_equal(tt, th0)
    s, tk, tt = O.extrapolate(th0, th2, g0, g1, 5, 1.0, 1e-3)
    np.testing.assert_array_equal(tt, tk)
    # inactive coordinates keep the observed two-step displacement
    inactive = np.abs(g0) <= float(np.float32(1e-3))
    assert inactive.sum() >= n // 5
    np.testing.assert_allclose(tk[inactive], th2[inactive], rtol=0, atol=1e-15)
    assert np.all(s[inactive] == 1.0)
    # K = 2 is the identity on the observed displacement everywhere
    s, tk, tt = O.extrapolate(th0, th2, g0, g1, 2, 1.0, 0.0)
    np.testing.assert_allclose(tk, th2, rtol=1e-13, atol=1e-15)
    # alpha blends linearly between theta_0 and theta_K
    s, tk, tt = O.extrapolate(th0, th2, g0, g1, 4, 0.3, 1e-3)
    np.testing.assert_allclose(tt, 0.7 * th0 + 0.3 * tk, rtol=1e-12, atol=1e-14)


def test_degenerate_and_clamped_ratio_readings():
    # r = -1 (S_2 = 0): keep the observed displacement
    assert O.scale_factor(1.5, -1.5, 4, 0.0) == 1.0
    assert O.scale_factor(1.5, -1.5, 5, 0.0) == 1.0
    # clamp: r = 10 with r_max = 2 behaves like r = 2
    assert O.scale_factor(1.0, 10.0, 4, 0.0, 2.0) == pytest.approx((1 - 2.0 ** 4) / (1 - 4.0))
    assert O.scale_factor(1.0, -10.0, 3, 0.0, 2.0) == pytest.approx((1 - (-2.0) ** 3) / (1 - 4.0))
    # clamping onto -1 lands on the degenerate rule
    assert O.scale_factor(1.0, -10.0, 4, 0.0, 1.0) == 1.0
    # r_max = inf is the printed rule
    assert O.scale_factor(1.0, 10.0, 3, 0.0) == pytest.approx(111.0 / 11.0)


# ---------------------------------------------------------------------------
# 3. Dense (non-diagonal) quadratics, d <= 4: brute-force K-step GD against the
#    oracle's theta_K, inside the bound the paper proves (Appendix A.5,
#    combined corollary with M_3 = 0), and the ratio-bias lemma (Appendix A.3).
# ---------------------------------------------------------------------------
def combined_bound(H, g0, eta, K, delta, R):
    """Right-hand side of the combined empirical-ratio bound for a quadratic
    loss (third derivative zero)."""
    Hoff = H - np.diag(np.diag(H))
    rho_max = max(1.0, np.linalg.norm(np.eye(len(H)) - eta * H, 2))
    A = np.abs(g0) > delta
    C = sum(n * R ** (n - 1) for n in range(1, K))
    D = 2 + sum(R ** n for n in range(K))
    t1 = K * (K - 1) / 2 * eta ** 2 * np.linalg.norm(Hoff, 2) * np.linalg.norm(g0) * rho_max ** (K - 2)
    t2 = eta ** 2 * C * np.abs(Hoff).sum(1).max() / delta * np.abs(g0).max() * np.linalg.norm(g0[A])
    t3 = eta * D * np.abs(g0[~A]).sum()
    t4 = eta ** 2 * np.abs((H @ g0)[~A]).sum()
    return t1 + t2 + t3 + t4


def bound_coefficients(K, eta):
    """Numeric coefficients of the five terms of the combined bound."""
    return {
        "coeff_offdiag": K * (K - 1) / 2 * eta ** 2,
        "coeff_active_ratio": eta ** 2,
        "coeff_inactive_mass": eta,
        "coeff_two_probe": eta ** 2,
        "coeff_nonquad": K * (K - 1) * (2 * K - 1) / 12 * eta ** 3,
        "rho_power_offdiag": K - 2,
        "rho_power_nonquad": K - 1,
    }


def read_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                k, v = line.split()
                out[k] = float(v)
    return out


def test_bound_helper_matches_printed_K3_illustration(golden_dir):
    g = read_golden(os.path.join(golden_dir, "bound_illustration_K3.txt"))
    got = bound_coefficients(int(g["K"]), g["eta"])
    for k, v in got.items():
        assert v == pytest.approx(g[k], rel=1e-12), k
    R = 2.0
    assert sum(n * R ** (n - 1) for n in range(1, 3)) == g["C_at_R2"]
    assert 2 + sum(R ** n for n in range(3)) == g["D_at_R2"]


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("K", [3, 4, 6])
def test_dense_quadratic_brute_force_within_paper_bound(seed, K):
    rng = np.random.default_rng(100 + seed)
    d = int(rng.integers(2, 5))
    Q = rng.normal(size=(d, d))
    H = np.diag(rng.uniform(0.5, 2.0, size=d)) + 0.05 * (Q + Q.T)      # SPD, weak coupling
    assert np.all(np.linalg.eigvalsh(H) > 0)
    eta = 0.05
    th0 = rng.normal(size=d)
    if seed % 2:
        th0[0] = np.linalg.solve(H, np.r_[1e-4, (H @ th0)[1:]])[0]    # nudge one gradient small
    grad = lambda th: H @ th
    g0 = grad(th0)
    th1 = th0 - eta * g0
    g1 = grad(th1)
    th2 = th1 - eta * g1
    delta = 1e-2
    scale, th_emp, _ = O.extrapolate(th0, th2, g0, g1, K, 1.0, delta)
    th_true = gd_unroll(th0, grad, eta, K)
    A = np.abs(g0) > float(np.float32(delta))
    rbar = 1 - eta * np.diag(H)
    r = g1 / g0
    R = max(np.abs(rbar).max(), np.abs(r[A]).max() if A.any() else 0.0)
    err = np.linalg.norm(th_emp - th_true)
    assert err <= combined_bound(H, g0, eta, K, float(np.float32(delta)), R) * (1 + 1e-9)
    # the error is real (the surrogate is not exact off the diagonal) ...
    assert err > 0
    # ... and the oracle's active displacement is -eta g0 S_K(r) with r from the
    # ratio-bias lemma: r_i = rbar_i - eta sum_{j != i} H_ij g0_j / g0_i
    Hoff = H - np.diag(np.diag(H))
    r_lemma = rbar - eta * (Hoff @ g0) / g0
    S_K = (1 - r_lemma ** K) / (1 - r_lemma)
    np.testing.assert_allclose((th_emp - th0)[A], (-eta * g0 * S_K)[A], rtol=1e-9, atol=1e-14)
    # inactive coordinates keep -eta (g0 + g1)
    np.testing.assert_allclose((th_emp - th0)[~A], (-eta * (g0 + g1))[~A], rtol=1e-12, atol=1e-16)


def test_diagonal_hessian_makes_the_surrogate_exact():
    rng = np.random.default_rng(7)
    d, eta, K = 4, 0.3, 7
    H = np.diag(rng.uniform(0.2, 3.0, size=d))
    th0 = rng.normal(size=d)
    g0 = H @ th0
    th1 = th0 - eta * g0
    g1 = H @ th1
    th2 = th1 - eta * g1
    _, tk, _ = O.extrapolate(th0, th2, g0, g1, K, 1.0, 0.0)
    np.testing.assert_allclose(tk, gd_unroll(th0, lambda t: H @ t, eta, K), rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------------------
# 4. OptimStep = AdamW: against a library AdamW in fp64 (Section 2 names AdamW
#    as the base optimizer; K = 2, alpha = 1 turns a GXPO step into three
#    consecutive AdamW steps on g0, g1, g_slow).
# ---------------------------------------------------------------------------
def torch_adamw_steps(theta0, grads, lr, betas, eps, wd):
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=lr, betas=betas, eps=eps, weight_decay=wd,
                            amsgrad=False, foreach=False)
    out = []
    for g in grads:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        out.append(p.detach().numpy().copy())
    st = opt.state[p]
    return out, st["exp_avg"].numpy().copy(), st["exp_avg_sq"].numpy().copy()


@pytest.mark.parametrize("wd,eps,lr", [(0.01, 1e-8, 1e-6), (0.1, 1e-3, 1e-2), (0.0, 1e-8, 3e-4)])
def test_adamw_optimstep_matches_library(wd, eps, lr):
    rng = np.random.default_rng(3)
    n = 1000
    th0 = rng.normal(scale=0.02, size=n)
    grads = [rng.normal(scale=0.05, size=n) for _ in range(7)]
    grads[2][::7] = 0.0
    cfg = O.OptimConfig("adamw", lr=lr, beta1=0.9, beta2=0.999, eps=eps, weight_decay=wd)
    m, v = np.zeros(n), np.zeros(n)
    th, cnt = th0.copy(), 0
    want, want_m, want_v = torch_adamw_steps(th0, grads, lr, (0.9, 0.999), eps, wd)
    for g, w in zip(grads, want):
        th, cnt = O.optim_step(cfg, cnt, th, g, m, v)
        np.testing.assert_allclose(th, w, rtol=1e-12, atol=1e-15)
        # the update itself, not just theta, must agree
        np.testing.assert_allclose(th - th0, w - th0, rtol=1e-9, atol=1e-16)
    np.testing.assert_allclose(m, want_m, rtol=1e-12, atol=1e-18)
    np.testing.assert_allclose(v, want_v, rtol=1e-12, atol=1e-20)
    assert cnt == 7


def test_gxpo_K2_alpha1_is_three_library_adamw_steps():
    rng = np.random.default_rng(4)
    n = 500
    th0 = rng.normal(scale=0.02, size=n)
    lr, wd, eps = 1e-3, 0.01, 1e-8
    cfg = O.GXPOConfig(optim=O.OptimConfig("adamw", lr=lr, eps=eps, weight_decay=wd),
                       K=2, alpha=1.0, delta=1e-8)
    orc = O.GXPOOracle(cfg, [th0])
    grads = []
    for step in range(3):
        g0, g1, gs = (rng.normal(scale=0.05, size=n) for _ in range(3))
        grads += [g0, g1, gs]
        orc.fast_step_1([g0])
        orc.fast_step_2([g1])
        orc.extrapolate([g0], [g1])
        orc.slow_step([gs])
        orc.gate_step()
    want, want_m, want_v = torch_adamw_steps(th0, grads, lr, (0.9, 0.999), eps, wd)
    np.testing.assert_allclose(orc.theta[0], want[-1], rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(orc.m[0], want_m, rtol=1e-12)
    np.testing.assert_allclose(orc.v[0], want_v, rtol=1e-12)
    assert orc.optim_steps == 9          # the step counter runs through all three steps


def test_parameter_groups_match_library_param_groups():
    """Per-tensor lr / weight-decay multipliers against a library AdamW with three parameter groups
    (decay, no decay, lower learning rate), K = 2 and alpha = 1 so that GXPO is three plain steps."""
    rng = np.random.default_rng(8)
    sizes = [300, 17, 120]
    lr, wd, eps = 1e-3, 0.1, 1e-8
    lr_scale, wd_scale = [1.0, 1.0, 0.25], [1.0, 0.0, 2.0]
    th0 = [rng.normal(scale=0.5, size=n) for n in sizes]
    cfg = O.GXPOConfig(optim=O.OptimConfig("adamw", lr=lr, eps=eps, weight_decay=wd), K=2, alpha=1.0, delta=1e-8)
    orc = O.GXPOOracle(cfg, th0)
    orc.lr_scale, orc.weight_decay_scale = lr_scale, wd_scale
    params = [torch.nn.Parameter(torch.tensor(t, dtype=torch.float64)) for t in th0]
    opt = torch.optim.AdamW([dict(params=[p], lr=lr * a, weight_decay=wd * b) for p, a, b in zip(params, lr_scale, wd_scale)],
                            betas=(0.9, 0.999), eps=eps, foreach=False)

    def lib_step(gs):
        for p, g in zip(params, gs):
            p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
    for step in range(2):
        g0, g1, gs = ([rng.normal(scale=0.05, size=n) for n in sizes] for _ in range(3))
        orc.fast_step_1(g0); lib_step(g0)
        orc.fast_step_2(g1); lib_step(g1)
        orc.extrapolate(g0, g1)
        orc.slow_step(gs); lib_step(gs)
        orc.gate_step()
    for i, p in enumerate(params):
        np.testing.assert_allclose(orc.theta[i], p.detach().numpy(), rtol=1e-11, atol=1e-15)
        np.testing.assert_allclose(orc.m[i], opt.state[p]["exp_avg"].numpy(), rtol=1e-12)
    # the groups really differ: tensor 1 saw no decay, tensor 2 a quarter of the step
    assert orc.optim_steps == 6


def test_optimizer_state_is_not_rolled_back_on_reposition():
    """With alpha = 0 the parameters return to theta^t before the slow step but
    the moments and the step counter keep what the two probes did."""
    rng = np.random.default_rng(5)
    n = 64
    th0 = rng.normal(size=n)
    g0, g1, gs = (rng.normal(size=n) for _ in range(3))
    lr = 1e-2
    cfg = O.GXPOConfig(optim=O.OptimConfig("adamw", lr=lr, weight_decay=0.0), K=4, alpha=0.0, delta=0.0)
    orc = O.GXPOOracle(cfg, [th0])
    orc.fast_step_1([g0]); orc.fast_step_2([g1]); orc.extrapolate([g0], [g1]); orc.slow_step([gs])
    # library: three AdamW steps give the moments; the third step's UPDATE applied at theta_0
    want, want_m, want_v = torch_adamw_steps(th0, [g0, g1, gs], lr, (0.9, 0.999), 1e-8, 0.0)
    third_update = want[2] - want[1]
    np.testing.assert_allclose(orc.theta[0], th0 + third_update, rtol=1e-9, atol=1e-14)
    np.testing.assert_allclose(orc.m[0], want_m, rtol=1e-12)


def test_multi_tensor_equals_flat():
    rng = np.random.default_rng(6)
    sizes = [5, 1, 33, 8]
    n = sum(sizes)
    th0 = rng.normal(size=n)
    gs = [rng.normal(size=n) for _ in range(3)]
    split = lambda a: np.split(a, np.cumsum(sizes)[:-1])
    cfg = O.GXPOConfig(K=5, alpha=0.5, delta=1e-3)
    flat, multi = O.GXPOOracle(cfg, [th0]), O.GXPOOracle(cfg, split(th0))
    for o, f in ((flat, lambda a: [a]), (multi, split)):
        o.fast_step_1(f(gs[0])); o.fast_step_2(f(gs[1])); o.extrapolate(f(gs[0]), f(gs[1]))
        o.slow_step(f(gs[2]))
    np.testing.assert_array_equal(np.concatenate(multi.theta), flat.theta[0])
    i1, i2 = flat.gate_step(), multi.gate_step()
    assert i1.norm == pytest.approx(i2.norm, rel=1e-15)
    assert i1.norm == pytest.approx(np.linalg.norm(gs[2]), rel=1e-14)
    np.testing.assert_allclose(multi.tensor_norms(), [np.linalg.norm(x) for x in split(gs[2])], rtol=1e-14)


# ---------------------------------------------------------------------------
# 5. Gate: numpy statistics, hand-computed cases, and the paper's printed
#    backward-pass budget (Section 2.3, Eq. (10) and the sentence after it).
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("ddof", [0, 1])
def test_gate_statistics_match_numpy(ddof):
    rng = np.random.default_rng(8)
    w = 6
    gate = O.RollingGate(O.GateConfig(tau=1e9, window=w, eps=1e-8, ddof=ddof, min_count=2))
    hist = []
    for t in range(25):
        x = float(rng.uniform(1, 2))
        info = gate.step(t, x)
        past = hist[-w:]
        if len(past) >= 2:
            assert info.evaluated
            assert info.mu == pytest.approx(np.mean(past), rel=1e-14)
            assert info.sigma == pytest.approx(np.std(past, ddof=ddof), rel=1e-12)
            assert info.z == pytest.approx((x - np.mean(past)) / (np.std(past, ddof=ddof) + 1e-8), rel=1e-10)
        else:
            assert not info.evaluated and not info.tripped
        hist.append(x)
    assert gate.s_star is None


def test_gate_hand_computed_threshold_is_inclusive_and_one_sided():
    # past norms 1, 3: mu = 2, population sigma = 1; eps = 0.5 -> Z = (5 - 2)/1.5 = 2 exactly
    mk = lambda tau: O.RollingGate(O.GateConfig(tau=tau, window=4, eps=0.5, ddof=0, min_count=2))
    g = mk(2.0)
    g.step(0, 1.0); g.step(1, 3.0)
    info = g.step(2, 5.0)
    assert (info.mu, info.sigma, info.z) == (2.0, 1.0, 2.0)
    assert info.tripped and info.s_star == 3                 # Z >= tau trips; s* = t + 1
    g = mk(2.0 + 1e-12)
    g.step(0, 1.0); g.step(1, 3.0)
    assert not g.step(2, 5.0).tripped
    g = mk(2.0)
    g.step(0, 1.0); g.step(1, 3.0)
    assert not g.step(2, -100.0).tripped                      # a drop never trips
    assert g.buffer == [1.0, 3.0, -100.0]                     # current norm inserted afterwards


def test_gate_warmup_window_and_permanence():
    g = O.RollingGate(O.GateConfig(tau=3.0, window=3, min_count=None))
    infos = [g.step(t, x) for t, x in enumerate([1.0, 1.1, 0.9, 1.0, 50.0, 1.0])]
    assert [i.evaluated for i in infos] == [False, False, False, True, True, True]
    assert [i.tripped for i in infos[:4]] == [False] * 4
    assert infos[4].tripped and infos[4].s_star == 5
    assert infos[5].s_star == 5                               # permanent
    assert g.buffer == [1.0, 50.0, 1.0]                       # window keeps the last w, trip included
    g2 = O.RollingGate(O.GateConfig(tau=3.0, window=3))
    g2.step(0, 1.0)
    assert g2.step(1, float("nan")).tripped                   # non-finite norm trips (reading)


def test_backward_pass_budget_matches_printed_table(golden_dir):
    """Drive Algorithm 1 for T = 300 steps with a norm sequence that jumps at a
    chosen step and count gradient hand-offs: the paper's table rows give
    total BP for each shutoff step, and Section 2.3 gives 3 s* + (T - s*)."""
    rows = []
    with open(os.path.join(golden_dir, "alpha_sensitivity_budget.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, a, s, bp = line.split()
                rows.append((int(k), float(a), int(s), int(bp)))
    assert len(rows) == 9
    T, n = 300, 16
    rng = np.random.default_rng(9)
    for K, alpha, shutoff, total_bp in sorted(set(rows)):
        cfg = O.GXPOConfig(optim=O.OptimConfig("adamw", lr=1e-7), K=K, alpha=alpha, delta=1e-8,
                           gate=O.GateConfig(tau=3.0, window=10))
        orc = O.GXPOOracle(cfg, [rng.normal(scale=0.02, size=n)])
        base = rng.normal(size=n)

        def grad_fn(ths, orc=orc, base=base, shutoff=shutoff):
            jitter = 1.0 + 1e-3 * math.sin(1.7 * orc.t)
            boost = 10.0 if orc.t >= shutoff - 1 else 1.0     # first unstable step is t = s* - 1
            return [base * jitter * boost]

        for _ in range(T):
            orc.train_step(grad_fn)
        assert orc.s_star == shutoff
        assert orc.backward_passes == total_bp == 3 * shutoff + (T - shutoff)
        assert orc.optim_steps == total_bp                   # one OptimStep per backward pass


# ---------------------------------------------------------------------------
# 6. bf16 rounding helper against the library conversion
# ---------------------------------------------------------------------------
def test_bf16_rounding_matches_library():
    rng = np.random.default_rng(10)
    x = np.concatenate([
        rng.normal(scale=0.02, size=4096), rng.normal(scale=1e3, size=256),
        np.array([0.0, -0.0, 1.0, -1.0, np.inf, -np.inf, 1e-40, 3.3895314e38, 65504.0]),
        # exact ties: 1 + 2^-8 (rounds to even, down) and 1 + 3*2^-8 (rounds up)
        np.array([1.00390625, 1.01171875, -1.00390625, -1.01171875]),
    ]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = O.bf16_round_bits(x)
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(O.bf16_bits_to_f64(got),
                                  torch.from_numpy(x).to(torch.bfloat16).double().numpy())


# ---------------------------------------------------------------------------
# 7. Mechanism diagnostics (appendix table of active-phase diagnostics): against
#    numpy definitions on random data and closed forms on the diagonal surrogate
# ---------------------------------------------------------------------------
def test_diagnostics_match_numpy_definitions():
    rng = np.random.default_rng(12)
    sizes = [300, 17, 1000]
    mk = lambda: [rng.normal(size=n) for n in sizes]
    th0, th2, g0, g1, gs = mk(), mk(), mk(), mk(), mk()
    g0[0][::7] = 1e-5                                    # some inactive coordinates
    K, delta, r_max = 5, 1e-3, 3.0
    d = O.diagnostics(th0, th2, g0, g1, gs, K, delta, r_max)
    cat = lambda l: np.concatenate(l)
    G0, G1, GS, T0, T2 = cat(g0), cat(g1), cat(gs), cat(th0), cat(th2)
    act = np.abs(G0) > float(np.float32(delta))
    r = np.clip(G1[act] / G0[act], -r_max, r_max)
    scale = np.ones_like(G0)
    scale[act] = np.array([O.scale_factor(a, b, K, delta, r_max) for a, b in zip(G0[act], G1[act])])
    assert d["norm_g0"] == pytest.approx(np.linalg.norm(G0), rel=1e-13)
    assert d["norm_g1"] == pytest.approx(np.linalg.norm(G1), rel=1e-13)
    assert d["norm_g_slow"] == pytest.approx(np.linalg.norm(GS), rel=1e-13)
    assert d["cos_g0_g_slow"] == pytest.approx(np.dot(G0, GS) / np.linalg.norm(G0) / np.linalg.norm(GS), rel=1e-11)
    assert d["retention_mean"] == pytest.approx(np.mean(r), rel=1e-12)
    assert d["retention_std"] == pytest.approx(np.std(r), rel=1e-12)
    assert d["scale_mean"] == pytest.approx(np.mean(scale[act]), rel=1e-12)
    assert d["inactive_fraction"] == pytest.approx(1 - act.mean(), rel=1e-12)
    assert d["inactive_fraction"] > 0.02
    assert d["displacement_ratio"] == pytest.approx(np.linalg.norm((T2 - T0) * scale) / np.linalg.norm(T2 - T0), rel=1e-12)


def test_diagnostics_closed_forms_on_the_diagonal_surrogate():
    """Plain GD on the diagonal quadratic: r_i = 1 - eta h_i exactly, so every statistic has a
    closed form; with alpha = 1 the corrective gradient is rho^K g0 coordinate-wise."""
    h, ts, th0 = surrogate_numpy()
    eta, K = 0.1, 4
    orc = O.GXPOOracle(gd_config(K, 1.0, eta), [th0])
    orc.train_step(lambda ths: [h * (ths[0] - ts)])
    d = orc.diagnostics()
    rho = 1 - eta * h
    g0 = h * (th0 - ts)
    S = lambda n: sum(rho ** j for j in range(n))
    assert d["retention_mean"] == pytest.approx(np.mean(rho), rel=1e-12)
    assert d["retention_std"] == pytest.approx(np.std(rho), rel=1e-10)
    assert d["scale_mean"] == pytest.approx(np.mean(S(K) / S(2)), rel=1e-12)
    assert d["inactive_fraction"] == 0.0
    assert d["displacement_ratio"] == pytest.approx(np.linalg.norm(g0 * S(K)) / np.linalg.norm(g0 * S(2)), rel=1e-11)
    assert d["norm_g1"] == pytest.approx(np.linalg.norm(rho * g0), rel=1e-12)
    gK = rho ** K * g0
    assert d["norm_g_slow"] == pytest.approx(np.linalg.norm(gK), rel=1e-11)
    assert d["cos_g0_g_slow"] == pytest.approx(np.dot(g0, gK) / np.linalg.norm(g0) / np.linalg.norm(gK), rel=1e-11)


# ---------------------------------------------------------------------------
# 8. Global-norm gradient clipping against the library routine
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("max_norm,scale", [(1.0, 0.05), (1.0, 5.0), (0.3, 1.0)])
def test_clipping_matches_library_clip_grad_norm(max_norm, scale):
    rng = np.random.default_rng(13)
    sizes = [40, 7, 300]
    grads = [rng.normal(scale=scale, size=n) for n in sizes]
    params = [torch.nn.Parameter(torch.zeros(n, dtype=torch.float64)) for n in sizes]
    for p, g in zip(params, grads):
        p.grad = torch.tensor(g)
    total = torch.nn.utils.clip_grad_norm_(params, max_norm)
    got, norm, c = O.clip_gradients(grads, max_norm)
    assert norm == pytest.approx(float(total), rel=1e-13)
    assert (c < 1.0) == (norm > max_norm)
    for g, p in zip(got, params):
        np.testing.assert_allclose(g, p.grad.numpy(), rtol=1e-12, atol=0)
    # the clipped gradient has norm max_norm (up to the 1e-6 guard) when clipping is active
    if c < 1.0:
        assert np.sqrt(sum(np.sum(g * g) for g in got)) == pytest.approx(max_norm, rel=1e-5)
    assert O.clip_gradients(grads, 0.0)[2] == 1.0


def test_clipped_gxpo_step_is_the_unclipped_step_on_clipped_gradients():
    """With clipping every OptimStep, the ratio included, sees c*g; the gate still sees ||g_slow||."""
    rng = np.random.default_rng(14)
    n, clip = 200, 1.0
    th0 = rng.normal(scale=0.02, size=n)
    g0, g1, gs = (rng.normal(scale=s, size=n) for s in (0.5, 0.02, 0.4))      # g0 and g_slow get clipped, g1 does not
    mk = lambda c: O.GXPOOracle(O.GXPOConfig(optim=O.OptimConfig("adamw", lr=1e-3), K=5, alpha=0.5, delta=1e-4, clip_norm=c), [th0])
    a, b = mk(clip), mk(0.0)
    cg = lambda g: O.clip_gradients([g], clip)[0][0]
    a.fast_step_1([g0]); a.fast_step_2([g1]); a.extrapolate([g0], [g1]); a.slow_step([gs]); ia = a.gate_step()
    b.fast_step_1([cg(g0)]); b.fast_step_2([cg(g1)]); b.extrapolate([cg(g0)], [cg(g1)]); b.slow_step([cg(gs)]); b.gate_step()
    np.testing.assert_array_equal(a.theta[0], b.theta[0])
    np.testing.assert_array_equal(a.m[0], b.m[0])
    assert ia.norm == pytest.approx(np.linalg.norm(gs), rel=1e-14) and ia.norm > clip


# ---------------------------------------------------------------------------
# 9. Explicit lookahead (n real fast steps, reposition, slow correction): on the
#    diagonal quadratic with plain GD it must land where the extrapolation lands
#    (the paper's corollary read the other way round), and where brute-force GD lands.
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("K", [2, 3, 5, 10])
@pytest.mark.parametrize("alpha", [1.0, 0.5])
def test_explicit_lookahead_equals_extrapolation_on_the_surrogate(K, alpha):
    h, ts, th0 = surrogate_numpy()
    eta = 0.1
    grad = lambda th: h * (th - ts)
    cfg_x = gd_config(K, alpha, eta)
    cfg_e = O.GXPOConfig(optim=O.OptimConfig("gd", lr=eta), K=K, alpha=alpha, delta=0.0, explicit_steps=K,
                         gate=O.GateConfig(tau=3.0, window=10))
    ox, oe = O.GXPOOracle(cfg_x, [th0]), O.GXPOOracle(cfg_e, [th0])
    for _ in range(3):
        start = oe.theta[0].copy()
        ox.train_step(lambda ths: [grad(ths[0])])
        th = oe.theta
        for j in range(K):
            th = oe.explicit_fast_step(j, [grad(th[0])])
        np.testing.assert_allclose(th[0], gd_unroll(start, grad, eta, K), rtol=1e-12, atol=1e-14)   # K real GD steps
        tt = oe.explicit_reposition()
        oe.slow_step([grad(tt[0])])
        oe.gate_step()
        np.testing.assert_allclose(oe.theta_tilde[0], ox.theta_tilde[0], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(oe.theta[0], ox.theta[0], rtol=1e-10, atol=1e-12)
    assert oe.backward_passes == 3 * (K + 1) and ox.backward_passes == 9     # K + 1 against 3 per step
    assert oe.optim_steps == 3 * (K + 1)
