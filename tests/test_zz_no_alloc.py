"""The entry point that allocates nothing (gxpo_slow_step_noalloc) against gxpo_slow_step on a
one-tensor context: same kernels, same order of additions, so every output must be bit-identical.
Two calls in a row, the second on a smaller input (the built-in workspace keeps the first call's
partials; none of them may leak into the second result)."""
import math

import pytest
import torch

from paper_2605_06755_amd import binding as B
from paper_2605_06755_amd import synth

pytestmark = pytest.mark.gpu


def reference_and_inputs(numel, cfg, seed, with_copy):
    """Runs one active step up to the reposition on a context, snapshots the state, lets the context take the
    slow step, and returns (snapshot, g_slow, optimizer step number of the slow step, results of the context)."""
    gdt = torch.float32 if cfg.grad_dtype == B.GXPO_GRAD_F32 else torch.bfloat16
    adam = cfg.optimizer == B.GXPO_OPT_ADAMW
    problem = synth.policy_problem(numel, seed=seed, sigma=0.05, device="cuda")
    bufs = dict(theta=problem.theta_0.clone(), theta_probe=torch.empty(numel, device="cuda"))
    if adam:
        bufs.update(m=torch.zeros(numel, device="cuda"), v=torch.zeros(numel, device="cuda"))
    if with_copy:
        bufs["model_copy"] = torch.zeros(numel, dtype=torch.bfloat16, device="cuda")
    ctx = B.gxpo_init(cfg, [bufs])
    noise = synth.step_noise(problem, 0)
    g = lambda th: synth.quadratic_grad(problem, th, noise, out_dtype=gdt)
    g0 = g(bufs["theta"]); B.gxpo_fast_steps(ctx, 0, [g0])
    g1 = g(bufs["theta_probe"]); B.gxpo_fast_steps(ctx, 1, [g1])
    B.gxpo_extrapolate(ctx, [g0], [g1])
    gs = g(bufs["theta"])
    torch.cuda.synchronize()
    snap = {k: v.clone() for k, v in bufs.items() if k != "theta_probe"}
    step_no = B.gxpo_get_state(ctx).optim_steps + 1
    B.gxpo_slow_step(ctx, [gs])
    info = B.gxpo_gate(ctx)
    want = {k: v.clone() for k, v in bufs.items() if k != "theta_probe"}
    B.gxpo_destroy(ctx)
    return snap, gs, step_no, want, info.norm


def bits(t):
    return t.view(torch.int32) if t.element_size() == 4 else t.view(torch.int16)


@pytest.mark.parametrize("optimizer,grad_dtype,with_copy", [("adamw", "f32", True), ("adamw", "bf16", False), ("gd", "f32", False)])
def test_noalloc_slow_step_equals_the_context_path_twice_in_a_row(optimizer, grad_dtype, with_copy):
    cfg = B.make_config(optimizer=optimizer, grad_dtype=grad_dtype, K=5, alpha=0.5, delta=1.75e-3,
                        lr=1e-3 if optimizer == "gd" else 1e-4, weight_decay=0.01, copy_mask=7)
    out = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    for numel, seed in ((3_000_003, 51), (70_001, 52)):          # 11719 blocks in two runs of partials, then 274 blocks
        snap, gs, step_no, want, norm = reference_and_inputs(numel, cfg, seed, with_copy)
        B.gxpo_slow_step_noalloc(cfg, snap, step_no, gs, out)
        torch.cuda.synchronize()
        for k in want:
            assert torch.equal(bits(snap[k]), bits(want[k])), f"numel {numel}: {k} differs from gxpo_slow_step's"
        assert math.sqrt(float(out)) == norm, f"numel {numel}: norm {math.sqrt(float(out))!r} vs {norm!r}"


def test_noalloc_refuses_what_it_cannot_hold():
    cfg = B.make_config(K=5, lr=1e-4)
    out = torch.zeros(1, dtype=torch.float64, device="cuda")
    n = 1024
    t = dict(theta=torch.zeros(n, device="cuda"), m=torch.zeros(n, device="cuda"), v=torch.zeros(n, device="cuda"))
    g = torch.zeros(n, device="cuda")
    # a size beyond the built-in workspace is refused on the host from the count alone (no buffer that large is touched)
    import ctypes
    rec = B.gxpo_tensor()
    rec.numel = B.GXPO_NOALLOC_MAX_NUMEL + 1
    rec.theta, rec.m, rec.v = t["theta"].data_ptr(), t["m"].data_ptr(), t["v"].data_ptr()
    rc = B._lib.gxpo_slow_step_noalloc(ctypes.byref(cfg), ctypes.byref(rec), 1, g.data_ptr(), out.data_ptr(), None)
    assert rc == B.GXPO_ERR_INVALID_ARG and "exceeds" in B.gxpo_last_error()
    with pytest.raises(B.GxpoError) as e:
        B.gxpo_slow_step_noalloc(B.make_config(K=5, lr=1e-4, clip_norm=1.0), t, 1, g, out)
    assert e.value.code == B.GXPO_ERR_UNSUPPORTED
    with pytest.raises(B.GxpoError) as e:
        B.gxpo_slow_step_noalloc(cfg, t, 0, g, out)                   # optimizer steps are numbered from 1
    assert e.value.code == B.GXPO_ERR_INVALID_ARG
    with pytest.raises(B.GxpoError) as e:
        B.gxpo_slow_step_noalloc(cfg, dict(t, m=t["theta"]), 1, g, out)   # m aliases theta
    assert e.value.code == B.GXPO_ERR_INVALID_ARG
    assert float(t["theta"].abs().sum()) == 0.0 and float(out) == 0.0      # nothing ran
