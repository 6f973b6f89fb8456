"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(fused second step, one wave per block, phased HBM layout).

The oracle cannot run 1.5e9 - 8e9 coordinates in seconds, but every step of the path is
per-coordinate, so it checks windows of coordinates (tensor heads and tails, block
boundaries, random interior windows) one by one; norms are checked on whole small tensors
by the oracle and at full size against an fp64 library reduction; gate decisions against
the oracle's gate fed with those independently computed norms.
"""
import math

import numpy as np
import pytest
import torch

from oracle import gxpo_oracle as O
from paper_2605_06755_amd import binding as B
from paper_2605_06755_amd import layout as layout_mod
from paper_2605_06755_amd import synth
from tests import gxpo_harness as H

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _release_cached_blocks():
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    yield
    gc.collect()
    torch.cuda.empty_cache()


def sumsq64(t: torch.Tensor, chunk: int = 1 << 27) -> float:
    """sum of squares in fp64 with a library reduction, chunked to bound temporaries"""
    total = 0.0
    for lo in range(0, t.numel(), chunk):
        total += float(t[lo:lo + chunk].double().square_().sum())
    return total


def need_memory(gib):
    free, _ = torch.cuda.mem_get_info()
    if free < gib * (1 << 30):
        pytest.skip(f"needs {gib} GiB of free HBM, {free / (1 << 30):.0f} available")


def windows_for(layout, rng, n_random, width=768):
    """(flat_start, length) windows: head and tail of every tensor (whole tensor if small),
    plus random interior windows that straddle block boundaries."""
    out, off = [], 0
    spans = []
    for _, n in layout:
        spans.append((off, n))
        off += -(-n // 4) * 4
    for start, n in spans:
        if n <= 2 * width:
            out.append((start, n))
        else:
            out.append((start, width))
            out.append((start + n - width, width))
    big = [(s, n) for s, n in spans if n > 4 * width]
    for _ in range(n_random):
        s, n = big[int(rng.integers(len(big)))]
        lo = int(rng.integers(width, n - 2 * width))
        out.append((s + lo - (lo % 256) + 200, width))         # starts 56 elements before a block boundary
    return out


def gather(flat, windows):
    idx = torch.cat([torch.arange(s, s + n, device=flat.device) for s, n in windows])
    return H.f64(flat[idx])


def dot64(a: torch.Tensor, b: torch.Tensor, chunk: int = 1 << 27) -> float:
    total = 0.0
    for lo in range(0, a.numel(), chunk):
        total += float((a[lo:lo + chunk].double() * b[lo:lo + chunk].double()).sum())
    return total


def count_active(g: torch.Tensor, delta32: float, chunk: int = 1 << 28) -> int:
    n = 0
    for lo in range(0, g.numel(), chunk):
        n += int((g[lo:lo + chunk].float().abs() > delta32).sum())
    return n


def run_sampled_active_step(spec_layout, *, seed, grad_dtype, with_copy, n_random, step_index=0, K=8, alpha=0.5, diagnostics=False,
                            clip_norm=0.0):
    dev = torch.device("cuda:0")
    numels = [n for _, n in spec_layout]
    padded = synth.padded_numel(spec_layout, 4)
    gdt = torch.float32 if grad_dtype == "f32" else torch.bfloat16
    flat, gflat = layout_mod.alloc_engine_state(padded, dev, adam=True, model_copy=with_copy, grad_dtype=gdt)
    views = {k: synth.split_like(v, spec_layout, 4) for k, v in flat.items()}
    g0, g1, gs = (synth.split_like(g, spec_layout, 4) for g in gflat)
    quad = synth.ChunkedQuadratic(padded, seed, 0.05, device=dev)
    quad.init_theta(flat["theta"])
    cfg = B.make_config(grad_dtype=grad_dtype, K=K, alpha=alpha, delta=1.75e-3, lr=1e-6, weight_decay=0.01,
                        tau=3.0, window=10, fuse_step2=True, copy_mask=7, diagnostics=diagnostics, clip_norm=clip_norm)
    ctx = B.gxpo_init(cfg, [{k: views[k][i] for k in views} for i in range(len(numels))])
    rng = np.random.default_rng(seed)
    wins = windows_for(spec_layout, rng, n_random)

    # a first, unchecked step so that m, v and the step counter are not trivial
    quad.grad(flat["theta"], 100, gflat[0]); B.gxpo_fast_steps(ctx, 0, g0)
    quad.grad(flat["theta_probe"], 100, gflat[1]); B.gxpo_fast_steps(ctx, 1, g1)
    B.gxpo_extrapolate(ctx, g0, g1)
    quad.grad(flat["theta"], 100, gflat[2]); B.gxpo_slow_step(ctx, gs)
    B.gxpo_gate(ctx)

    st = B.gxpo_get_state(ctx)
    oc = H.oracle_config(cfg)
    oc.clip_norm = 0.0          # the oracle sees windows only: it is handed gradients already clipped with the whole list's norm
    orc = O.GXPOOracle(oc, [gather(flat["theta"], wins)])
    orc.m, orc.v, orc.optim_steps = [gather(flat["m"], wins)], [gather(flat["v"], wins)], st.optim_steps
    start = orc.theta[0].copy()

    def clipped(sample, whole_list):
        if not clip_norm:
            return sample
        c = O.clip_coefficient(math.sqrt(sum(sumsq64(x) for x in whole_list)), clip_norm)
        assert c < 0.9, "the threshold was meant to bite"
        return sample * c

    def check(key, ref, label, amplified=False):
        got = gather(flat[key], wins)
        extra = 4.0 * 2.0 ** -24 * np.abs(ref) * cfg.alpha * np.abs(orc.scale[0]) if amplified else None
        if amplified and clip_norm:
            extra = extra + cfg.alpha * np.abs(orc._theta_2[0] - orc._theta_0[0]) * orc.scale[0] ** 2 * 2.0 ** -22
        H.assert_close(got, ref, label, extra_abs=extra)
        if key in ("theta", "theta_probe"):
            num = np.linalg.norm((got - start) - (ref - start))
            den = np.linalg.norm(ref - start)
            floor = (2.0 + cfg.alpha * cfg.K) * 2.0 ** -24 * np.linalg.norm(ref)
            assert num <= 1e-4 * den + floor, f"{label}: displacement error {num:.3e} of {den:.3e}"

    quad.grad(flat["theta"], step_index, gflat[0])
    B.gxpo_fast_steps(ctx, 0, g0)
    g0s = clipped(gather(gflat[0], wins), g0)
    check("theta_probe", orc.fast_step_1([g0s])[0], "theta^{t,1}")
    quad.grad(flat["theta_probe"], step_index, gflat[1])
    B.gxpo_fast_steps(ctx, 1, g1)
    g1s = clipped(gather(gflat[1], wins), g1)
    orc.fast_step_2([g1s])
    B.gxpo_extrapolate(ctx, g0, g1)
    ref_t = orc.extrapolate([g0s], [g1s])[0]
    check("theta", ref_t, "theta~", amplified=True)
    check("m", orc.m[0], "m after step 2"); check("v", orc.v[0], "v after step 2")
    if with_copy:
        bits = flat["model_copy"][torch.cat([torch.arange(s, s + n, device=dev) for s, n in wins])]
        got_bits = bits.cpu().view(torch.int16).numpy().view(np.uint16)
        th32 = flat["theta"][torch.cat([torch.arange(s, s + n, device=dev) for s, n in wins])].cpu().numpy()
        np.testing.assert_array_equal(got_bits, O.bf16_round_bits(th32))
        H.assert_close(O.bf16_bits_to_f64(got_bits), ref_t, "bf16 copy at theta~", rtol=H.RTOL_BF16)
    quad.grad(flat["theta"], step_index, gflat[2])
    B.gxpo_slow_step(ctx, gs)
    gss = clipped(gather(gflat[2], wins), gs)
    ref_n = orc.slow_step([gss])[0]
    check("theta", ref_n, "theta^{t+1}", amplified=True)
    check("m", orc.m[0], "m after slow step"); check("v", orc.v[0], "v after slow step")
    info = B.gxpo_gate(ctx)
    # norms: full size against an fp64 library reduction, small tensors against the oracle
    want = math.sqrt(sum(sumsq64(x) for x in gs))
    assert info.norm == pytest.approx(want, rel=1e-11)
    tn = B.gxpo_tensor_norms(ctx)
    assert math.sqrt(sum(x * x for x in tn)) == pytest.approx(info.norm, rel=1e-12)
    small = [i for i, n in enumerate(numels) if n <= (1 << 22)][:80]
    for i in small:
        assert tn[i] == pytest.approx(math.sqrt(O.sum_squares(H.f64(gs[i]))), rel=1e-12), f"tensor {i} norm"
    st2 = B.gxpo_get_state(ctx)
    assert (st2.t, st2.optim_steps, st2.backward_passes) == (st.t + 1, st.optim_steps + 3, st.backward_passes + 3)
    if diagnostics:
        # the whole-list statistics that have a definition a library reduction can evaluate at this size
        d = B.gxpo_get_diagnostics(ctx)
        n0 = math.sqrt(sum(sumsq64(x) for x in g0))
        n1 = math.sqrt(sum(sumsq64(x) for x in g1))
        assert d.norm_g0 == pytest.approx(n0, rel=1e-11) and d.norm_g1 == pytest.approx(n1, rel=1e-11)
        assert d.norm_g_slow == pytest.approx(want, rel=1e-11)
        cos = sum(dot64(a, b) for a, b in zip(g0, gs)) / (n0 * want)
        assert d.cos_g0_g_slow == pytest.approx(cos, rel=1e-9)
        active = sum(count_active(x, float(np.float32(cfg.delta))) for x in g0)
        assert d.inactive_fraction == pytest.approx(1.0 - active / sum(numels), rel=1e-12, abs=1e-15)
        # and on the sampled coordinates the oracle's statistics bracket what the engine reports for the whole list
        ref = orc.diagnostics()
        assert abs(d.retention_mean - ref["retention_mean"]) < 0.05 and abs(d.scale_mean - ref["scale_mean"]) < 0.2
        assert d.displacement_ratio == pytest.approx(ref["displacement_ratio"], rel=0.05)
    B.gxpo_destroy(ctx)
    return info


def test_config2_qwen_1p5b_flat_full_size():
    need_memory(70)
    info = run_sampled_active_step([("flat", synth.QWEN25_1P5B_PARAMS)], seed=1, grad_dtype="f32", with_copy=False, n_random=400)
    assert 1900 < info.norm < 2100           # ~ sqrt(P) * 0.05 plus the curvature term


def test_config3_qwen_7b_flat_with_bf16_copy_full_size():
    need_memory(235)
    run_sampled_active_step([("flat", synth.QWEN25_7B_PARAMS)], seed=2, grad_dtype="f32", with_copy=True, n_random=400)


def test_config4_llama_8b_ragged_bf16_grads_full_size():
    need_memory(200)
    layout = synth.llama31_8b_layout()
    assert len(layout) == 290 and sum(n for _, n in layout) == 8_030_257_152
    run_sampled_active_step(layout, seed=3, grad_dtype="bf16", with_copy=False, n_random=300)


@pytest.mark.parametrize("clip_norm", [0.0, 1000.0])
def test_config2_full_size_periodic_data_every_accumulator(clip_norm):
    """Every buffer of the 1.54e9-parameter workload is a 4e6-element pattern repeated 385 times.  All of
    the path is per-coordinate apart from sums, so the engine's full-size result must be the oracle's
    result on ONE period, repeated (bit-identical from period to period), every mean, fraction and ratio
    of the diagnostics must equal the one-period value and every norm sqrt(385) times it.  That checks all
    ten reduction accumulators, the clipping pre-passes and the block plan at the benchmark's size."""
    need_memory(70)
    dev = torch.device("cuda:0")
    P, period = synth.QWEN25_1P5B_PARAMS, 4_000_000
    reps = P // period
    assert reps * period == P and reps == 385
    problem = synth.policy_problem(period, seed=12, sigma=0.05, device=dev)
    flat, gflat = layout_mod.alloc_engine_state(P, dev, adam=True, grad_dtype=torch.float32)
    tiled = lambda t: t.view(reps, period)
    tiled(flat["theta"]).copy_(problem.theta_0)
    cfg = B.make_config(K=5, alpha=0.5, delta=1.75e-3, lr=1e-4, weight_decay=0.01, tau=3.0, window=10, gate_min_count=2,
                        fuse_step2=True, diagnostics=1, clip_norm=clip_norm)
    ctx = B.gxpo_init(cfg, [dict(flat)])
    oc = H.oracle_config(cfg)
    oc.clip_norm = clip_norm / math.sqrt(reps)           # one period carries 1/385 of the squared norm
    orc = O.GXPOOracle(oc, [H.f64(problem.theta_0)])
    g0, g1, gs = ([g] for g in gflat)

    def fill(gbuf, theta_period, step):
        g = synth.quadratic_grad(problem, theta_period, synth.step_noise(problem, step))
        tiled(gbuf).copy_(g)
        return [H.f64(g)]

    def check_state(label, theta_extra):
        for k, ref in (("theta", orc.theta), ("m", orc.m), ("v", orc.v)):
            rows = tiled(flat[k])
            for r in (1, reps // 2, reps - 1):
                assert torch.equal(rows[r], rows[0]), f"{label}: {k} differs between periods 0 and {r}"
            H.assert_close(H.f64(rows[0]), ref[0], f"{label} {k}", extra_abs=theta_extra if k == "theta" else None)

    for step in range(2):
        a0 = fill(gflat[0], flat["theta"][:period], step)
        B.gxpo_fast_steps(ctx, 0, g0)
        th1 = orc.fast_step_1(a0)
        H.assert_close(H.f64(flat["theta_probe"][:period]), th1[0], f"step {step} theta^(t,1)")
        a1 = fill(gflat[1], flat["theta_probe"][:period], step)
        B.gxpo_fast_steps(ctx, 1, g1)
        orc.fast_step_2(a1)
        B.gxpo_extrapolate(ctx, g0, g1)
        ref_t = orc.extrapolate(a0, a1)
        extra = 4.0 * 2.0 ** -24 * np.abs(ref_t[0]) * cfg.alpha * np.abs(orc.scale[0])
        if clip_norm:
            extra = extra + cfg.alpha * np.abs(orc._theta_2[0] - orc._theta_0[0]) * orc.scale[0] ** 2 * 2.0 ** -22
        H.assert_close(H.f64(flat["theta"][:period]), ref_t[0], f"step {step} theta~", extra_abs=extra)
        a_s = fill(gflat[2], flat["theta"][:period], step)
        B.gxpo_slow_step(ctx, gs)
        orc.slow_step(a_s)
        info, ref_info = B.gxpo_gate(ctx), orc.gate_step()
        check_state(f"step {step} after the slow step", extra)
        assert info.norm == pytest.approx(math.sqrt(reps) * ref_info.norm, rel=1e-12)
        got, ref = B.gxpo_get_diagnostics(ctx), orc.diagnostics()
        for k in ("norm_g0", "norm_g1", "norm_g_slow"):
            ref[k] *= math.sqrt(reps)
        H.check_diagnostics(got, ref, aliased=False, what=f"full-size periodic step {step} clip={clip_norm}")
        if clip_norm:
            assert ref["norm_g0"] > 1.5 * clip_norm          # the threshold bites
        # the next step starts from the engine's own state
        orc.theta, orc.m, orc.v = [H.f64(flat["theta"][:period])], [H.f64(flat["m"][:period])], [H.f64(flat["v"][:period])]
    B.gxpo_destroy(ctx)


def test_tensor_longer_than_2_to_32_elements_inside_a_list():
    """Element offsets inside a tensor are 64-bit: a 2^32 + 1027 element tensor between two small ones
    (the table-driven path, unlike the flat 7.6e9 buffer, which takes its pointers from the kernel arguments)."""
    need_memory(150)
    layout = [("head", 4099), ("long", (1 << 32) + 1027), ("tail", 257)]
    run_sampled_active_step(layout, seed=8, grad_dtype="f32", with_copy=False, n_random=300)


def test_config4_llama_8b_with_gradient_clipping_full_size():
    """Clipping on the ragged list at full size: the norm pre-passes run over 290 tensors of bf16 gradients, the
    factor never leaves the device; the oracle is handed the sampled gradients clipped with the norm of the whole list."""
    need_memory(200)
    run_sampled_active_step(synth.llama31_8b_layout(), seed=7, grad_dtype="bf16", with_copy=False, n_random=300, clip_norm=2000.0)


def test_config4_llama_8b_with_diagnostics_full_size():
    """The ragged 290-tensor list at full size with every accumulator on: norms, cosine and the active count
    against fp64 library reductions over the whole list, the rest against the oracle on the sampled windows."""
    need_memory(200)
    run_sampled_active_step(synth.llama31_8b_layout(), seed=6, grad_dtype="bf16", with_copy=False, n_random=300, diagnostics=True)


@pytest.mark.parametrize("K,alpha", [(3, 0.1), (5, 1.0), (10, 0.5)])
def test_lora_shaped_many_small_tensors_paper_grid(K, alpha):
    """224 rank-128 adapter tensors (the paper's Qwen2.5-7B runs train LoRA adapters on q, k, v, o),
    at the paper's own lookahead depths and reposition strengths."""
    layout = synth.qwen25_7b_lora_layout()
    assert len(layout) == 224 and sum(n for _, n in layout) == 80_740_352
    run_sampled_active_step(layout, seed=5, grad_dtype="f32", with_copy=False, n_random=200, K=K, alpha=alpha)


def test_config5_gate_transition_full_size():
    """3.2e9 parameters, 50 steps, sigma 0.05 -> 1.0 at step 30: every gate decision must equal
    the oracle gate's decision on independently computed norms; after the trip the engine is
    in the fallback phase and the fallback step equals the first fast step bit for bit on a
    window and the oracle within tolerance."""
    need_memory(100)
    dev = torch.device("cuda:0")
    P = synth.GATE_STRESS_PARAMS
    layout = [("flat", P)]
    flat, gflat = layout_mod.alloc_engine_state(P, dev, adam=True, grad_dtype=torch.float32)
    quad = synth.ChunkedQuadratic(P, 4, 0.05, device=dev)
    quad.init_theta(flat["theta"])
    cfg = B.make_config(K=8, alpha=0.5, delta=1.75e-3, lr=1e-6, weight_decay=0.01, tau=3.0, window=10)
    ctx = B.gxpo_init(cfg, [dict(flat)])
    gate = O.RollingGate(H.oracle_config(cfg).gate)
    g0, g1, gs = ([g] for g in gflat)
    rng = np.random.default_rng(4)
    wins = windows_for(layout, rng, 200)
    n_active = 0
    for step in range(50):
        sig = 0.05 if step < 30 else 1.0
        st = B.gxpo_get_state(ctx)
        if st.s_star < 0 or st.t < st.s_star:
            n_active += 1
            quad.grad(flat["theta"], step, gflat[0], sig); B.gxpo_fast_steps(ctx, 0, g0)
            quad.grad(flat["theta_probe"], step, gflat[1], sig); B.gxpo_fast_steps(ctx, 1, g1)
            B.gxpo_extrapolate(ctx, g0, g1)
            quad.grad(flat["theta"], step, gflat[2], sig); B.gxpo_slow_step(ctx, gs)
            info = B.gxpo_gate(ctx)
            want_norm = math.sqrt(sumsq64(gflat[2]))
            assert info.norm == pytest.approx(want_norm, rel=1e-11)
            ref = gate.step(step, want_norm)
            assert bool(info.evaluated) == ref.evaluated and bool(info.tripped) == ref.tripped, f"step {step}"
            if ref.evaluated:
                assert info.z == pytest.approx(ref.z, rel=1e-5, abs=1e-5)
            if info.tripped and step < 30:                     # chance trip: agree, re-arm both
                st = B.gxpo_get_state(ctx); st.s_star = -1; B.gxpo_set_state(ctx, st)
                gate.s_star = None
        else:
            # fallback phase: check one step on windows against the oracle
            pre = {k: gather(flat[k], wins) for k in ("theta", "m", "v")}
            quad.grad(flat["theta"], step, gflat[0], sig)
            B.gxpo_fallback_step(ctx, g0)
            if step == 31:
                orc = O.GXPOOracle(H.oracle_config(cfg), [pre["theta"]])
                orc.m, orc.v, orc.optim_steps = [pre["m"]], [pre["v"]], st.optim_steps
                orc.gate.s_star, orc.t = 0, 1
                ref = orc.fallback_step([gather(gflat[0], wins)])[0]
                got = gather(flat["theta"], wins)
                H.assert_close(got, ref, "fallback theta")
                H.assert_close(gather(flat["m"], wins), orc.m[0], "fallback m")
                H.assert_close(gather(flat["v"], wins), orc.v[0], "fallback v")
                num = np.linalg.norm((got - pre["theta"]) - (ref - pre["theta"]))
                assert num <= 1e-4 * np.linalg.norm(ref - pre["theta"]) + 2.0 ** -24 * np.linalg.norm(ref)
    st = B.gxpo_get_state(ctx)
    assert st.s_star == 31 and gate.s_star == 31 and n_active == 31 and st.t == 50
    assert st.backward_passes == 3 * 31 + 19 and st.optim_steps == 3 * 31 + 19
    B.gxpo_destroy(ctx)
