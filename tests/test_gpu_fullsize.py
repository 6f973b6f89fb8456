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


MIN_DENSE = 1 << 26          # coordinates the oracle checks one by one at full size
GROUPS = 8                   # the sample is checked in this many groups, one host thread each


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


def dense_windows(layout, rng, total=MIN_DENSE, width=1 << 17):
    """Heads, tails and short block-straddling windows as in windows_for, plus enough long random
    windows (each starting 56 elements before a block boundary) to reach `total` coordinates.
    Long windows are drawn per tensor in proportion to its size, so every large tensor is hit."""
    out = windows_for(layout, rng, 64)
    have = sum(n for _, n in out)
    spans, off = [], 0
    for _, n in layout:
        spans.append((off, n))
        off += -(-n // 4) * 4
    big = [(s, n) for s, n in spans if n > 4 * width]
    if not big:                                               # a list of small tensors: take them whole
        return [(s, n) for s, n in spans]
    weights = np.array([n for _, n in big], dtype=np.float64)
    weights /= weights.sum()
    while have < total:
        s, n = big[int(rng.choice(len(big), p=weights))]
        lo = int(rng.integers(256, n - width - 256))
        out.append((s + lo - (lo % 256) + 200, width))
        have += width
    return out


def gather(flat, windows):
    """The windows of a flat device buffer as one host float64 array (exact widening)."""
    return H.f64(torch.cat([flat[s:s + n] for s, n in windows]))


def gather_raw(flat, windows):
    return torch.cat([flat[s:s + n] for s, n in windows]).cpu()


def split_groups(windows, k=GROUPS):
    """k lists of windows with about the same number of coordinates each."""
    order = sorted(windows, key=lambda w: -w[1])
    groups, load = [[] for _ in range(k)], [0] * k
    for w in order:
        i = load.index(min(load))
        groups[i].append(w)
        load[i] += w[1]
    return [g for g in groups if g]


def in_threads(fn, items):
    """fn(item) for every item, one host thread each (the C oracle and numpy release the interpreter
    lock); the first failure is re-raised."""
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=len(items)) as pool:
        return list(pool.map(fn, items))


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


class SampleGroup:
    """One group of sampled windows with its own oracle, stepped beside the engine."""

    def __init__(self, wins, flat, cfg, oc, optim_steps):
        self.wins, self.cfg = wins, cfg
        self.count = sum(n for _, n in wins)
        self.orc = O.GXPOOracle(oc, [gather(flat["theta"], wins)])
        self.orc.m, self.orc.v, self.orc.optim_steps = [gather(flat["m"], wins)], [gather(flat["v"], wins)], optim_steps
        self.start = self.orc.theta[0].copy()

    def check(self, flat, key, ref, label, amplified=False, clip_norm=0.0):
        cfg, orc = self.cfg, self.orc
        got = gather(flat[key], self.wins)
        extra = 4.0 * 2.0 ** -24 * np.abs(ref) * cfg.alpha * np.abs(orc.scale[0]) if amplified else None
        if amplified and clip_norm:
            extra = extra + cfg.alpha * np.abs(orc._theta_2[0] - orc._theta_0[0]) * orc.scale[0] ** 2 * 2.0 ** -22
        H.assert_close(got, ref, label, extra_abs=extra)
        if key in ("theta", "theta_probe"):
            num = np.linalg.norm((got - self.start) - (ref - self.start))
            den = np.linalg.norm(ref - self.start)
            floor = (2.0 + cfg.alpha * cfg.K) * 2.0 ** -24 * np.linalg.norm(ref)
            assert num <= 1e-4 * den + floor, f"{label}: displacement error {num:.3e} of {den:.3e}"

    def check_copy(self, flat, ref, label, key="theta"):
        got_bits = gather_raw(flat["model_copy"].view(torch.int16), self.wins).numpy().view(np.uint16)
        th32 = gather_raw(flat[key], self.wins).numpy()
        np.testing.assert_array_equal(got_bits, O.bf16_round_bits(th32), err_msg=label)
        H.assert_close(O.bf16_bits_to_f64(got_bits), ref, label, rtol=H.RTOL_BF16)


def run_sampled_active_step(spec_layout, *, seed, grad_dtype, with_copy, step_index=0, K=8, alpha=0.5, diagnostics=False,
                            clip_norm=0.0, total=MIN_DENSE, alternating=False):
    """One active step at full size in bench.py's launch configuration; at least `total` coordinates
    (all tensor heads and tails, block-straddling windows, long random windows) are compared with
    the oracle one by one after every call.  `alternating`: with the second buffer set (bench.py --alternating);
    theta~, m, v are then looked for in theta_probe, m_alt, v_alt."""
    TH2, M2, V2 = ("theta_probe", "m_alt", "v_alt") if alternating else ("theta", "m", "v")
    dev = torch.device("cuda:0")
    numels = [n for _, n in spec_layout]
    padded = synth.padded_numel(spec_layout, 4)
    gdt = torch.float32 if grad_dtype == "f32" else torch.bfloat16
    flat, gflat = layout_mod.alloc_engine_state(padded, dev, adam=True, model_copy=with_copy, grad_dtype=gdt, alternating=alternating)
    assert ("m_alt" in flat) == alternating
    views = {k: synth.split_like(v, spec_layout, 4) for k, v in flat.items()}
    g0, g1, gs = (synth.split_like(g, spec_layout, 4) for g in gflat)
    quad = synth.ChunkedQuadratic(padded, seed, 0.05, device=dev)
    quad.init_theta(flat["theta"])
    cfg = B.make_config(grad_dtype=grad_dtype, K=K, alpha=alpha, delta=1.75e-3, lr=1e-6, weight_decay=0.01,
                        tau=3.0, window=10, fuse_step2=True, copy_mask=7, diagnostics=diagnostics, clip_norm=clip_norm)
    ctx = B.gxpo_init(cfg, [{k: views[k][i] for k in views} for i in range(len(numels))])
    rng = np.random.default_rng(seed)
    wins = dense_windows(spec_layout, rng, total)
    n_checked = sum(n for _, n in wins)
    assert n_checked >= min(total, sum(numels)), f"only {n_checked} coordinates sampled"

    # a first, unchecked step so that m, v and the step counter are not trivial
    quad.grad(flat["theta"], 100, gflat[0]); B.gxpo_fast_steps(ctx, 0, g0)
    quad.grad(flat["theta_probe"], 100, gflat[1]); B.gxpo_fast_steps(ctx, 1, g1)
    B.gxpo_extrapolate(ctx, g0, g1)
    quad.grad(flat[TH2], 100, gflat[2]); B.gxpo_slow_step(ctx, gs)
    B.gxpo_gate(ctx)

    st = B.gxpo_get_state(ctx)
    oc = H.oracle_config(cfg)
    oc.clip_norm = 0.0          # the oracle sees windows only: it is handed gradients already clipped with the whole list's norm
    groups = [SampleGroup(w, flat, cfg, oc, st.optim_steps) for w in split_groups(wins)]

    def clip_of(whole_list):
        if not clip_norm:
            return 1.0
        c = O.clip_coefficient(math.sqrt(sum(sumsq64(x) for x in whole_list)), clip_norm)
        assert c < 0.9, "the threshold was meant to bite"
        return c

    quad.grad(flat["theta"], step_index, gflat[0])
    B.gxpo_fast_steps(ctx, 0, g0)
    c0 = clip_of(g0)

    def after_fast_1(grp):
        grp.g0 = gather(gflat[0], grp.wins) * c0
        grp.check(flat, "theta_probe", grp.orc.fast_step_1([grp.g0])[0], "theta^{t,1}")
    in_threads(after_fast_1, groups)

    quad.grad(flat["theta_probe"], step_index, gflat[1])
    B.gxpo_fast_steps(ctx, 1, g1)
    c1 = clip_of(g1)
    B.gxpo_extrapolate(ctx, g0, g1)

    def after_extrapolate(grp):
        grp.g1 = gather(gflat[1], grp.wins) * c1
        grp.orc.fast_step_2([grp.g1])
        ref_t = grp.orc.extrapolate([grp.g0], [grp.g1])[0]
        grp.check(flat, TH2, ref_t, "theta~", amplified=True, clip_norm=clip_norm)
        grp.check(flat, M2, grp.orc.m[0], "m after step 2")
        grp.check(flat, V2, grp.orc.v[0], "v after step 2")
        if with_copy:
            grp.check_copy(flat, ref_t, "bf16 copy at theta~", TH2)
    assert B.gxpo_get_state(ctx).current_set == (1 if alternating else 0)
    in_threads(after_extrapolate, groups)

    quad.grad(flat[TH2], step_index, gflat[2])
    B.gxpo_slow_step(ctx, gs)
    cs = clip_of(gs)

    def after_slow(grp):
        ref_n = grp.orc.slow_step([gather(gflat[2], grp.wins) * cs])[0]
        grp.check(flat, "theta", ref_n, "theta^{t+1}", amplified=True, clip_norm=clip_norm)
        grp.check(flat, "m", grp.orc.m[0], "m after slow step")
        grp.check(flat, "v", grp.orc.v[0], "v after slow step")
        if with_copy:
            grp.check_copy(flat, ref_n, "bf16 copy at theta^{t+1}")
    in_threads(after_slow, groups)

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
        ref = groups[0].orc.diagnostics()
        assert abs(d.retention_mean - ref["retention_mean"]) < 0.05 and abs(d.scale_mean - ref["scale_mean"]) < 0.2
        assert d.displacement_ratio == pytest.approx(ref["displacement_ratio"], rel=0.05)
    B.gxpo_destroy(ctx)
    return info, n_checked


def test_config2_qwen_1p5b_flat_full_size():
    need_memory(70)
    info, n = run_sampled_active_step([("flat", synth.QWEN25_1P5B_PARAMS)], seed=1, grad_dtype="f32", with_copy=False)
    assert n >= MIN_DENSE
    assert 1900 < info.norm < 2100           # ~ sqrt(P) * 0.05 plus the curvature term


def test_config2_full_size_with_alternating_state():
    """bench.py --alternating: the second buffer set in another DRAM rank, every pass out of place."""
    need_memory(90)
    info, n = run_sampled_active_step([("flat", synth.QWEN25_1P5B_PARAMS)], seed=11, grad_dtype="f32", with_copy=False, alternating=True)
    assert n >= MIN_DENSE


def test_config3_qwen_7b_flat_with_bf16_copy_full_size():
    need_memory(235)
    _, n = run_sampled_active_step([("flat", synth.QWEN25_7B_PARAMS)], seed=2, grad_dtype="f32", with_copy=True)
    assert n >= MIN_DENSE


def test_config4_llama_8b_ragged_bf16_grads_full_size():
    need_memory(200)
    layout = synth.llama31_8b_layout()
    assert len(layout) == 290 and sum(n for _, n in layout) == 8_030_257_152
    _, n = run_sampled_active_step(layout, seed=3, grad_dtype="bf16", with_copy=False)
    assert n >= MIN_DENSE


def assert_every_period_equals_the_first(rows: torch.Tensor, label: str):
    """rows: (reps, period) view of a device buffer; every row must equal row 0 bit for bit (compared on the
    device as raw bits, 2^27 elements at a time to bound temporaries)."""
    bits = rows.view(torch.int32) if rows.element_size() == 4 else rows.view(torch.int16)
    first = bits[0:1]
    chunk_rows = max(1, (1 << 27) // bits.shape[1])
    for lo in range(0, bits.shape[0], chunk_rows):
        same = (bits[lo:lo + chunk_rows] == first).all(dim=1)
        if not bool(same.all()):
            bad = lo + int((~same).nonzero()[0])
            raise AssertionError(f"{label} differs between periods 0 and {bad}")


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
            assert_every_period_equals_the_first(rows, f"{label}: {k}")
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


def run_periodic_list(layout, period, *, seed, grad_dtype, with_copy, steps=2, K=5, alpha=0.5, lr=1e-4):
    """Every tensor of `layout` holds its own `period`-element pattern, repeated.  Apart from sums the path is
    per-coordinate, so after every call each tensor must be bit-identical from period to period -- checked on the
    device over ALL periods -- and one period per tensor must match the oracle, which runs the list of patterns;
    norms follow from the repeat counts.  Covers every block of the full-size launch."""
    dev = torch.device("cuda:0")
    numels = [n for _, n in layout]
    assert all(n % period == 0 for n in numels) and period % 4 == 0
    T, reps = len(layout), [n // period for n in numels]
    gdt = torch.float32 if grad_dtype == "f32" else torch.bfloat16
    problem = synth.policy_problem(period * T, seed=seed, sigma=0.05, device=dev)      # tensor t's pattern is slice t
    flat, gflat = layout_mod.alloc_engine_state(sum(numels), dev, adam=True, model_copy=with_copy, grad_dtype=gdt)
    views = {k: synth.split_like(v, layout, 4) for k, v in flat.items()}
    g0, g1, gs = (synth.split_like(g, layout, 4) for g in gflat)
    sl = lambda x, t: x[t * period:(t + 1) * period]
    tiled = lambda view: view.view(-1, period)
    for t in range(T):
        tiled(views["theta"][t]).copy_(sl(problem.theta_0, t))
    cfg = B.make_config(grad_dtype=grad_dtype, K=K, alpha=alpha, delta=1.75e-3, lr=lr, weight_decay=0.01, tau=3.0, window=10,
                        gate_min_count=2, fuse_step2=True, copy_mask=7)
    ctx = B.gxpo_init(cfg, [{k: views[k][i] for k in views} for i in range(T)])
    orc = O.GXPOOracle(H.oracle_config(cfg), [H.f64(sl(problem.theta_0, t)) for t in range(T)])
    first_rows = lambda key: torch.cat([views[key][t][:period] for t in range(T)])

    def fill(gviews, theta_patterns, step):
        g = synth.quadratic_grad(problem, theta_patterns, synth.step_noise(problem, step)).to(gdt)
        for t in range(T):
            tiled(gviews[t]).copy_(sl(g, t))
        return [H.f64(sl(g, t)) for t in range(T)]

    def check(key, refs, label, extras=None, periodic=True):
        for t in range(T):
            if periodic:
                assert_every_period_equals_the_first(tiled(views[key][t]), f"{label}: {key} of tensor {t}")
            H.assert_close(H.f64(views[key][t][:period]), refs[t], f"{label}: {key} of tensor {t}",
                           extra_abs=None if extras is None else extras[t])

    def check_copy(refs, label):
        for t in range(T):
            rows = tiled(views["model_copy"][t])
            assert_every_period_equals_the_first(rows, f"{label}: model_copy of tensor {t}")
            got_bits = rows[0].cpu().view(torch.int16).numpy().view(np.uint16)
            np.testing.assert_array_equal(got_bits, O.bf16_round_bits(views["theta"][t][:period].cpu().numpy()), err_msg=label)
            H.assert_close(O.bf16_bits_to_f64(got_bits), refs[t], f"{label}: bf16 copy of tensor {t}", rtol=H.RTOL_BF16)

    for step in range(steps):
        a0 = fill(g0, first_rows("theta"), step)
        B.gxpo_fast_steps(ctx, 0, g0)
        check("theta_probe", orc.fast_step_1(a0), f"step {step} theta^(t,1)")
        a1 = fill(g1, first_rows("theta_probe"), step)
        B.gxpo_fast_steps(ctx, 1, g1)
        orc.fast_step_2(a1)
        B.gxpo_extrapolate(ctx, g0, g1)
        ref_t = orc.extrapolate(a0, a1)
        extras = [4.0 * 2.0 ** -24 * np.abs(r) * cfg.alpha * np.abs(sc) for r, sc in zip(ref_t, orc.scale)]
        check("theta", ref_t, f"step {step} theta~", extras)
        if with_copy:
            check_copy(ref_t, f"step {step} theta~")
        a_s = fill(gs, first_rows("theta"), step)
        B.gxpo_slow_step(ctx, gs)
        ref_n = orc.slow_step(a_s)
        info, ref_info = B.gxpo_gate(ctx), orc.gate_step()
        check("theta", ref_n, f"step {step} theta^(t+1)", extras)
        check("m", orc.m, f"step {step} m")
        check("v", orc.v, f"step {step} v")
        if with_copy:
            check_copy(ref_n, f"step {step} theta^(t+1)")
        ref_tn = orc.tensor_norms()
        for got, ref, r in zip(B.gxpo_tensor_norms(ctx), ref_tn, reps):
            assert got == pytest.approx(math.sqrt(r) * ref, rel=1e-12)
        assert info.norm == pytest.approx(math.sqrt(sum(r * x * x for r, x in zip(reps, ref_tn))), rel=1e-12)
        assert not info.tripped and not ref_info.tripped
        # the next step starts from the engine's own state
        orc.theta = [H.f64(views["theta"][t][:period]) for t in range(T)]
        orc.m = [H.f64(views["m"][t][:period]) for t in range(T)]
        orc.v = [H.f64(views["v"][t][:period]) for t in range(T)]
    B.gxpo_destroy(ctx)


def test_config3_full_size_periodic_data_with_bf16_copy():
    """7.6e9 parameters, all 1900 periods of every buffer (the bf16 copy included) compared on the device."""
    need_memory(235)
    P = synth.QWEN25_7B_PARAMS
    assert P % 4_000_000 == 0
    run_periodic_list([("flat", P)], 4_000_000, seed=13, grad_dtype="f32", with_copy=True)


def test_config4_full_size_periodic_data_per_tensor():
    """The 290-tensor Llama-3.1-8B list with bf16 gradients: every tensor repeats its own 4096-element pattern, so
    a block that read or wrote another tensor's data, or another offset, would break a period somewhere."""
    need_memory(200)
    run_periodic_list(synth.llama31_8b_layout(), 4096, seed=14, grad_dtype="bf16", with_copy=False)


def test_tensor_longer_than_2_to_32_elements_inside_a_list():
    """Element offsets inside a tensor are 64-bit: a 2^32 + 1027 element tensor between two small ones
    (the table-driven path, unlike the flat 7.6e9 buffer, which takes its pointers from the kernel arguments)."""
    need_memory(150)
    layout = [("head", 4099), ("long", (1 << 32) + 1027), ("tail", 257)]
    _, n = run_sampled_active_step(layout, seed=8, grad_dtype="f32", with_copy=False)
    assert n >= MIN_DENSE


def test_config4_llama_8b_with_gradient_clipping_full_size():
    """Clipping on the ragged list at full size: the norm pre-passes run over 290 tensors of bf16 gradients, the
    factor never leaves the device; the oracle is handed the sampled gradients clipped with the norm of the whole list."""
    need_memory(200)
    run_sampled_active_step(synth.llama31_8b_layout(), seed=7, grad_dtype="bf16", with_copy=False, clip_norm=2000.0)


def test_config4_llama_8b_with_diagnostics_full_size():
    """The ragged 290-tensor list at full size with every accumulator on: norms, cosine and the active count
    against fp64 library reductions over the whole list, the rest against the oracle on the sampled windows."""
    need_memory(200)
    run_sampled_active_step(synth.llama31_8b_layout(), seed=6, grad_dtype="bf16", with_copy=False, diagnostics=True)


@pytest.mark.parametrize("K,alpha", [(3, 0.1), (5, 1.0), (10, 0.5)])
def test_lora_shaped_many_small_tensors_paper_grid(K, alpha):
    """224 rank-128 adapter tensors (the paper's Qwen2.5-7B runs train LoRA adapters on q, k, v, o),
    at the paper's own lookahead depths and reposition strengths."""
    layout = synth.qwen25_7b_lora_layout()
    assert len(layout) == 224 and sum(n for _, n in layout) == 80_740_352
    _, n = run_sampled_active_step(layout, seed=5, grad_dtype="f32", with_copy=False, K=K, alpha=alpha, total=1 << 25)
    assert n >= 1 << 25


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
    wins = dense_windows(layout, rng)
    assert sum(n for _, n in wins) >= MIN_DENSE
    win_groups = split_groups(wins)
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
            # fallback phase: one step is checked against the oracle on the dense sample
            if step == 31:
                pre = [{k: gather(flat[k], w) for k in ("theta", "m", "v")} for w in win_groups]
            quad.grad(flat["theta"], step, gflat[0], sig)
            B.gxpo_fallback_step(ctx, g0)
            if step == 31:
                def check_fallback(i):
                    w, p = win_groups[i], pre[i]
                    orc = O.GXPOOracle(H.oracle_config(cfg), [p["theta"]])
                    orc.m, orc.v, orc.optim_steps = [p["m"]], [p["v"]], st.optim_steps
                    orc.gate.s_star, orc.t = 0, 1
                    ref = orc.fallback_step([gather(gflat[0], w)])[0]
                    got = gather(flat["theta"], w)
                    H.assert_close(got, ref, "fallback theta")
                    H.assert_close(gather(flat["m"], w), orc.m[0], "fallback m")
                    H.assert_close(gather(flat["v"], w), orc.v[0], "fallback v")
                    num = np.linalg.norm((got - p["theta"]) - (ref - p["theta"]))
                    assert num <= 1e-4 * np.linalg.norm(ref - p["theta"]) + 2.0 ** -24 * np.linalg.norm(ref)
                in_threads(check_fallback, list(range(len(win_groups))))
                del pre
    st = B.gxpo_get_state(ctx)
    assert st.s_star == 31 and gate.s_star == 31 and n_active == 31 and st.t == 50
    assert st.backward_passes == 3 * 31 + 19 and st.optim_steps == 3 * 31 + 19
    B.gxpo_destroy(ctx)


def test_rank_aware_placement_changes_no_result():
    """Buffers assembled from 512 MiB physical chunks (HIP virtual-memory API) and placed by DRAM rank are ordinary
    contiguous device arrays: the same inputs give bit-identical theta, m, v, bf16 copy and norm as plain allocations,
    data written through torch reads back, and every tensor spans several mapped chunks (so the library's range check
    walks adjacent mappings, and blocks straddle chunk boundaries)."""
    from paper_2605_06755_amd import hbm_arena
    need_memory(60)
    dev = torch.device("cuda:0")
    numel = 300_000_004                                   # 1.2 GB per fp32 buffer: three chunks each, ragged last block
    results = {}
    for placement in ("phased", "ranked", "ranked, alternating state"):
        alternating = placement.endswith("alternating state")
        try:
            flat, gflat = layout_mod.alloc_engine_state(numel, dev, adam=True, model_copy=True, grad_dtype=torch.bfloat16,
                                                        placement=placement.split(",")[0], alternating=alternating)
        except hbm_arena.ArenaUnavailable as e:
            pytest.skip(f"virtual-memory API not available: {e}")
        assert layout_mod.last_placement()["kind"] == placement.split(",")[0]
        assert ("m_alt" in flat and "v_alt" in flat) == alternating
        if placement != "phased":                         # scattered order, and theta, m, v of every chunk position chosen by measurement
            detail = layout_mod.last_placement()["detail"]
            assert detail["order"] == "scattered" and detail["tuned"]["positions"] == 3 and detail["tuned"]["candidates"] > 1
            assert detail["tuned"]["chosen_gbps"] >= detail["tuned"]["mean_gbps"] and detail["alternating"] == alternating
        for k, t in list(flat.items()) + [(f"g{i}", g) for i, g in enumerate(gflat)]:
            assert t.is_contiguous() and t.numel() == numel and t.device.type == "cuda", k
            assert t.data_ptr() % 65536 == {"m": 32768, "v": 32768, "m_alt": 32768, "v_alt": 32768, "g1": 1024}.get(k, 0), k
        if alternating:
            assert not bool(flat["m_alt"].any()) and not bool(flat["v_alt"].any())
        quad = synth.ChunkedQuadratic(numel, 9, 0.05, device=dev)
        quad.init_theta(flat["theta"])
        quad_first = synth.ChunkedQuadratic(numel, 9, 0.05, device=dev).chunk_problem(0).theta_0[:1 << 20]
        assert torch.equal(flat["theta"][:1 << 20], quad_first)                        # written through torch, read back
        cfg = B.make_config(grad_dtype="bf16", K=8, alpha=0.5, delta=1.75e-3, lr=1e-4, weight_decay=0.01, copy_mask=7)
        ctx = B.gxpo_init(cfg, [dict(flat)])
        quad.grad(flat["theta"], 0, gflat[0]); B.gxpo_fast_steps(ctx, 0, [gflat[0]])
        quad.grad(flat["theta_probe"], 0, gflat[1]); B.gxpo_fast_steps(ctx, 1, [gflat[1]])
        B.gxpo_extrapolate(ctx, [gflat[0]], [gflat[1]])
        assert B.gxpo_get_state(ctx).current_set == (1 if alternating else 0)          # theta~ is in the other set now
        quad.grad(flat["theta_probe" if alternating else "theta"], 0, gflat[2]); B.gxpo_slow_step(ctx, [gflat[2]])
        info = B.gxpo_gate(ctx)
        assert B.gxpo_get_state(ctx).current_set == 0
        keep = ("theta", "m", "v", "model_copy") + (() if alternating else ("theta_probe",))
        results[placement] = ({k: flat[k].clone() for k in keep}, info.norm)
        B.gxpo_destroy(ctx)
        del flat, gflat, quad, ctx
        import gc
        gc.collect()
        torch.cuda.empty_cache()
    a, na = results["phased"]
    for placement in ("ranked", "ranked, alternating state"):
        b, nb = results[placement]
        assert na == nb, placement
        for k in b:
            w = torch.int16 if k == "model_copy" else torch.int32
            assert torch.equal(a[k].view(w), b[k].view(w)), f"{k} depends on the placement ({placement})"
