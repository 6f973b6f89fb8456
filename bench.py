#!/usr/bin/env python3
"""GXPO active-step throughput on one MI355X.

One "step" is one whole active step of the update engine over every parameter:
gxpo_fast_steps(0), gxpo_fast_steps(1), gxpo_extrapolate (second fast step fused
in), gxpo_slow_step (+ sum of squares) and gxpo_gate.  The three gradient buffers
are produced once, before the timed region, by the synthetic trainer at the
points the algorithm asks for them (theta, theta^{t,1}, theta~) and are then
reused: computing gradients is the trainer's work, not the engine's.

Prints ONE JSON line.  `value`, `config`, `roofline` and `cpu_baseline` belong to
the headline workload (configs[1], the one the metric is quoted on).  Without
`--workload` the same timed loop is then run on the other large configurations
(configs[2], [3], [4]; for [4] also the fallback step) and reported under
`workloads`; `--workload X` measures X alone (that is what the profiles use).
"""
from __future__ import annotations

import argparse
import gc
import hashlib
import json
import math
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published peak
HEADLINE = "c2"
ALSO = ["c5", "c4", "c3"]       # the other large configurations, measured after the headline


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None, choices=["c1", "c2", "c3", "c4", "c4flat", "c5", "lora"],
                    help="measure this workload alone (default: configs[1] as the headline, then configs[2..4] under 'workloads')")
    ap.add_argument("--unfused", action="store_true", help="run the second fast step and the extrapolation as two passes")
    ap.add_argument("--same-phase", action="store_true", help="plain torch allocations instead of the phased HBM layout")
    ap.add_argument("--arena", action="store_true", help="carve all buffers from one plain allocation")
    ap.add_argument("--placement", default="auto", choices=["auto", "ranked", "ranked-scatter", "ranked-adjacent", "phased"],
                    help="ranked: rank-aware placement through HIP's virtual-memory API; phased: one plain allocation per buffer")
    ap.add_argument("--phases", default="", help="experiment: KiB phases (mod 64) of theta,theta_probe,m,v,g0,g1,g2[,model_copy]")
    ap.add_argument("--alternating", action="store_true",
                    help="two buffer sets (theta_probe, m_alt, v_alt next to theta, m, v; 8 B/param more) that every pass alternates "
                         "between instead of updating in place")
    ap.add_argument("--no-probe", action="store_true",
                    help="workloads with a bf16 model copy: deliver theta^{t,1} through the copy only (no fp32 theta_probe)")
    ap.add_argument("--explicit-steps", type=int, default=0, help="explicit lookahead with this many real fast steps instead of GXPO")
    ap.add_argument("--clip-norm", type=float, default=0.0, help="global-norm gradient clipping threshold (0 = off)")
    ap.add_argument("--diagnostics", action="store_true", help="also accumulate the mechanism diagnostics in the passes")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=1 << 28, help="elements of the workload the oracle is timed on")
    return ap.parse_args()


def workload_spec(name: str):
    from paper_2605_06755_amd import synth
    if name == "c1":
        return dict(label="plain-GD quadratic surrogate, 1,048,576 fp32 params, GD eta=0.1, K=4",
                    layout=[("flat", 1 << 20)], optimizer="gd", grad_dtype="f32", copy=False, seed=0,
                    cfg=dict(K=4, alpha=1.0, delta=0.0, lr=0.1), surrogate=True)
    if name == "c2":
        return dict(label="Qwen2.5-1.5B-sized flat fp32 buffer, P=1.54e9, AdamW, K=8, alpha=0.5, tau=3, w=10",
                    layout=[("flat", synth.QWEN25_1P5B_PARAMS)], optimizer="adamw", grad_dtype="f32", copy=False, seed=1,
                    cfg=dict(K=8, alpha=0.5, delta=1.75e-3, lr=1e-6))
    if name == "c3":
        return dict(label="Qwen2.5-7B-sized flat fp32 buffer, P=7.6e9, AdamW, bf16 model copy rewritten 3x per step",
                    layout=[("flat", synth.QWEN25_7B_PARAMS)], optimizer="adamw", grad_dtype="f32", copy=True, seed=2,
                    cfg=dict(K=8, alpha=0.5, delta=1.75e-3, lr=1e-6))
    if name == "c4":
        return dict(label="Llama-3.1-8B ragged layout, 290 tensors, P=8.03e9, bf16 grads, fp32 state",
                    layout=synth.llama31_8b_layout(), optimizer="adamw", grad_dtype="bf16", copy=False, seed=3,
                    cfg=dict(K=8, alpha=0.5, delta=1.75e-3, lr=1e-6))
    if name == "c4flat":
        return dict(label="the Llama-3.1-8B workload's 8.03e9 parameters as ONE flat tensor, bf16 grads (shows what the ragged list costs)",
                    layout=[("flat", sum(n for _, n in synth.llama31_8b_layout()))], optimizer="adamw", grad_dtype="bf16", copy=False,
                    seed=3, cfg=dict(K=8, alpha=0.5, delta=1.75e-3, lr=1e-6))
    if name == "c5":
        return dict(label="gate-transition buffer, flat fp32, P=3.2e9, AdamW; active and fallback steps",
                    layout=[("flat", synth.GATE_STRESS_PARAMS)], optimizer="adamw", grad_dtype="f32", copy=False, seed=4,
                    cfg=dict(K=8, alpha=0.5, delta=1.75e-3, lr=1e-6))
    if name == "lora":
        return dict(label="LoRA rank-128 adapters on q,k,v,o of a Qwen2.5-7B-shaped model: 224 small tensors, P=8.07e7",
                    layout=synth.qwen25_7b_lora_layout(), optimizer="adamw", grad_dtype="f32", copy=False, seed=5,
                    cfg=dict(K=10, alpha=0.5, delta=1.75e-3, lr=1e-6))
    raise ValueError(name)


def workload_title(name: str, spec) -> str:
    return (f"configs[{int(name[1]) - 1}]: " if name[0] == "c" and name[1:].isdigit() else "") + spec["label"]


def bytes_per_param(spec, fused: bool):
    """Algorithmic HBM bytes per parameter of each pass (reads + writes of every
    operand exactly once)."""
    g = 4 if spec["grad_dtype"] == "f32" else 2
    mv = 8 if spec["optimizer"] == "adamw" else 0          # m and v, read; the same again written
    c = 2 if spec["copy"] else 0
    step = 4 + mv + g + 4 + mv                                # theta, m, v, g in; theta, m, v out
    out = {"slow_step": step + c, "fallback_step": step + c}
    if fused:
        # probe pass: theta, m, v, g0 in; theta^{t,1} out (fp32 unless only the bf16 copy is wanted)
        out["fast_step_1"] = 4 + mv + g + (0 if spec.get("no_probe") else 4) + c
        # fused pass: theta, m, v, g0, g1 in; theta~, m, v out
        out["fused_steps_extrapolate"] = 4 + mv + g + g + 4 + mv + c
    else:
        out["fast_step_1"] = step + c
        out["fast_step_2"] = step
        out["extrapolate"] = 4 + 4 + g + g + 4 + c
    return out


def measure(name: str, args, want_cpu_inputs: bool = False):
    """Allocates the workload's buffers, runs the live step, the warm-up and the timed loop, returns the
    measurements and releases everything again."""
    import torch
    from paper_2605_06755_amd import binding as B
    from paper_2605_06755_amd import layout as layout_mod
    from paper_2605_06755_amd import synth

    dev = torch.device("cuda:0")
    spec = workload_spec(name)
    fused = not args.unfused and not args.explicit_steps
    if args.no_probe:
        if not (spec["copy"] and fused):
            print("bench.py: --no-probe needs a workload with a bf16 model copy and the fused schedule", file=sys.stderr)
            sys.exit(2)
        spec["no_probe"] = True
    layout = spec["layout"]
    numels = [n for _, n in layout]
    P = sum(numels)
    padded = synth.padded_numel(layout, 4)
    adam = spec["optimizer"] == "adamw"
    gdt = torch.float32 if spec["grad_dtype"] == "f32" else torch.bfloat16

    phases = None
    if args.phases:
        names = ["theta", "theta_probe", "m", "v", "g0", "g1", "g2", "model_copy"]
        phases = {n: float(x) for n, x in zip(names, args.phases.split(","))}
    # ---- device buffers (caller-owned), placed as paper_2605_06755_amd/layout.py describes ----------------
    if args.same_phase:
        flat = {"theta": torch.empty(padded, dtype=torch.float32, device=dev),
                "theta_probe": torch.empty(padded, dtype=torch.float32, device=dev)}
        if adam:
            flat["m"] = torch.zeros(padded, dtype=torch.float32, device=dev)
            flat["v"] = torch.zeros(padded, dtype=torch.float32, device=dev)
        if spec["copy"]:
            flat["model_copy"] = torch.empty(padded, dtype=torch.bfloat16, device=dev)
        gflat = [torch.empty(padded, dtype=gdt, device=dev) for _ in range(3)]
        placement = {"kind": "same-phase", "detail": None}
    else:
        # on request: two buffer sets the passes alternate between (8 B/param more HBM), where the schedule allows and they fit
        alternating = args.alternating and adam and fused and not spec.get("no_probe") and not args.arena
        kw = dict(adam=adam, model_copy=spec["copy"], grad_dtype=gdt, arena=args.arena, phases_kib=phases, placement=args.placement,
                  probe_is_read=not fused, verbose=True)
        try:
            flat, gflat = layout_mod.alloc_engine_state(padded, dev, alternating=alternating, **kw)
        except Exception as e:
            if not alternating:
                raise
            print(f"[{name}] no room for the second set of moments ({type(e).__name__}: {e}); updating in place", file=sys.stderr)
            gc.collect()
            torch.cuda.empty_cache()
            flat, gflat = layout_mod.alloc_engine_state(padded, dev, **kw)
        placement = layout_mod.last_placement()
    print(f"[{name}] base addresses:", {k: hex(v.data_ptr()) for k, v in flat.items()}, [hex(g.data_ptr()) for g in gflat], file=sys.stderr)
    views = {k: synth.split_like(v, layout, 4) for k, v in flat.items()}
    g0, g1, gs = (synth.split_like(g, layout, 4) for g in gflat)
    tensors = [{k: views[k][i] for k in views if not (spec.get("no_probe") and k == "theta_probe")}
               for i in range(len(numels))]

    if spec.get("surrogate"):
        quad = synth.ChunkedQuadratic(padded, spec["seed"], 0.0, h_dist="uniform", h_lo=0.1, h_hi=1.0, theta_std=1.0, device=dev)
    else:
        quad = synth.ChunkedQuadratic(padded, spec["seed"], 0.05, device=dev)
    quad.init_theta(flat["theta"])

    cfg = B.make_config(optimizer=spec["optimizer"], grad_dtype=spec["grad_dtype"], fuse_step2=fused, copy_mask=7,
                        window=10, tau=3.0, weight_decay=0.01,
                        diagnostics=args.diagnostics, clip_norm=args.clip_norm, explicit_steps=args.explicit_steps,
                        **spec["cfg"])
    ctx = B.gxpo_init(cfg, tensors)

    # ---- one live step: gradients evaluated where Algorithm 1 asks for them ----------------------------
    quad.grad(flat["theta"], 0, gflat[0])
    B.gxpo_fast_steps(ctx, 0, g0)
    quad.grad(flat["model_copy"].float() if spec.get("no_probe") else flat["theta_probe"], 0, gflat[1])
    B.gxpo_fast_steps(ctx, 1, g1)
    for j in range(2, args.explicit_steps):
        B.gxpo_fast_steps(ctx, j, g1)
    if args.explicit_steps:
        B.gxpo_extrapolate(ctx)
    else:
        B.gxpo_extrapolate(ctx, g0, g1)
    # with alternating state theta~ is in the other set's parameter buffer (gxpo_state.current_set)
    quad.grad(flat["theta_probe" if B.gxpo_get_state(ctx).current_set else "theta"], 0, gflat[2])
    B.gxpo_slow_step(ctx, gs)
    live_info = B.gxpo_gate(ctx)

    # the gradient buffers are the same every step: marshal their pointer lists once
    g0, g1, gs = B.GradList(ctx, g0), B.GradList(ctx, g1), B.GradList(ctx, gs)

    if args.explicit_steps:
        calls = tuple((f"fast_step_{j + 1}", (lambda j=j: B.gxpo_fast_steps(ctx, j, g0 if j == 0 else g1)))
                      for j in range(args.explicit_steps))
        calls += (("reposition", lambda: B.gxpo_extrapolate(ctx)), ("slow_step", lambda: B.gxpo_slow_step(ctx, gs)))
    else:
        calls = (("fast_step_1", lambda: B.gxpo_fast_steps(ctx, 0, g0)),
                 ("fast_step_2", lambda: B.gxpo_fast_steps(ctx, 1, g1)),
                 ("fused_steps_extrapolate" if fused else "extrapolate", lambda: B.gxpo_extrapolate(ctx, g0, g1)),
                 ("slow_step", lambda: B.gxpo_slow_step(ctx, gs)))

    def active_step(events=None, step_events=None):
        # events are recorded on torch's current stream, which is the stream the binding launches on
        if step_events is not None:
            a = torch.cuda.Event(enable_timing=True)
            a.record()
        for cname, fn in calls:
            if events is None or (fused and cname == "fast_step_2" and not args.clip_norm > 0):
                fn()
                continue
            ka, kb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ka.record()
            fn()
            kb.record()
            events.setdefault(cname, []).append((ka, kb))
        if step_events is not None:
            b = torch.cuda.Event(enable_timing=True)
            b.record()
            step_events.append((a, b))
        return B.gxpo_gate(ctx)

    # the interpreter's cyclic collector is not part of the path: a full collection (tens of ms with torch
    # loaded) landing inside the timed region would leave the GPU idle behind the gate's synchronisation
    gc.collect()
    gc.disable()
    for _ in range(args.warmup):
        active_step()
    torch.cuda.synchronize()
    events, step_events = {}, []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        info = active_step(events, step_events)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    gc.enable()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    step_ms = [a.elapsed_time(b) for a, b in step_events]
    kernel_ms = {k: statistics.median(a.elapsed_time(b) for a, b in v) for k, v in events.items()}
    kernel_ms_mean = {k: sum(a.elapsed_time(b) for a, b in v) / len(v) for k, v in events.items()}
    bpp = bytes_per_param(spec, fused)
    if args.explicit_steps:
        full = bpp["slow_step"]
        bpp = {f"fast_step_{j + 1}": full for j in range(args.explicit_steps)}
        bpp.update(reposition=12 + (2 if spec["copy"] else 0), slow_step=full, fallback_step=full)
    gbytes = 4 if spec["grad_dtype"] == "f32" else 2
    if args.diagnostics:
        bpp["slow_step"] += gbytes                                            # g0 read again for <g0, g_slow>
    if args.clip_norm > 0:
        if fused:
            bpp["fast_step_2"] = 0                                            # nothing but the norm pre-pass of g1 runs there
        for k in ("fast_step_1", "fast_step_2", "slow_step", "fallback_step"):   # norm pre-pass: the gradient is read twice
            if k in bpp:
                bpp[k] += gbytes
    step_bpp = sum(bpp[k] for k in kernel_ms)
    kernels = {k: {"ms": round(ms, 4), "ms_mean": round(kernel_ms_mean[k], 4), "bytes_per_param": bpp[k],
                   "gbps": round(bpp[k] * P / ms / 1e6, 1), "frac_of_peak": round(bpp[k] * P / ms / 1e6 / HBM_PEAK_GBPS, 4)}
               for k, ms in kernel_ms.items()}
    dominant = max(kernel_ms, key=lambda k: bpp[k])

    # ---- plain copy on the same box, same access pattern (context for the roofline fraction) ------------
    n_copy = min(padded, 1 << 30)
    for _ in range(2):
        B.gxpo_stream_copy(flat["theta_probe"][:n_copy], flat["theta"][:n_copy])
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(10):
        B.gxpo_stream_copy(flat["theta_probe"][:n_copy], flat["theta"][:n_copy])
    b.record()
    torch.cuda.synchronize()
    copy_gbps = 8.0 * n_copy * 10 / a.elapsed_time(b) / 1e6
    for k in kernels.values():
        k["frac_of_copy"] = round(k["gbps"] / copy_gbps, 4)

    # ---- fallback-phase throughput (reported for the gate-transition workload) ---------------------------
    fallback = None
    if name == "c5":
        st = B.gxpo_get_state(ctx)
        st.s_star = st.t
        B.gxpo_set_state(ctx, st)
        # with alternating state the steps read the two sets in turn; the gradient buffer next to each set is used
        # (the third buffer lies next to the second set), as a trainer with two gradient buffers would
        two_sets = "m_alt" in flat
        for i in range(args.warmup + args.warmup % 2):
            B.gxpo_fallback_step(ctx, gs if two_sets and i % 2 else g0)
        torch.cuda.synchronize()
        fev = []
        tf0 = time.perf_counter()
        for i in range(args.steps):
            fa, fb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            fa.record()
            B.gxpo_fallback_step(ctx, gs if two_sets and i % 2 else g0)
            fb.record()
            fev.append((fa, fb))
        torch.cuda.synchronize()
        fms = (time.perf_counter() - tf0) * 1e3 / args.steps
        fmed = statistics.median(x.elapsed_time(y) for x, y in fev)
        fallback = {"ms_per_step": round(fms, 4), "ms_per_step_median_events": round(fmed, 4), "gparams_per_s": round(P / fms / 1e6, 2),
                    "bytes_per_param": bpp["fallback_step"], "gbps": round(bpp["fallback_step"] * P / fms / 1e6, 1),
                    "frac_of_peak": round(bpp["fallback_step"] * P / fms / 1e6 / HBM_PEAK_GBPS, 4)}

    hbm_layout = describe_layout(placement, "m_alt" in flat)
    res = {
        "workload": workload_title(name, spec), "params": P, "tensors": len(numels), "grad_dtype": spec["grad_dtype"],
        "fused_step2": fused, "hbm_layout": hbm_layout, "bytes_per_param_per_step": step_bpp,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_median_events": round(statistics.median(step_ms), 4),
        "ms_per_step_min_max_events": [round(min(step_ms), 4), round(max(step_ms), 4)],
        "gparams_per_s": round(P / ms_per_step / 1e6, 3),
        "hbm_gbps_step": round(step_bpp * P / ms_per_step / 1e6, 1),
        "hbm_frac_of_peak_step": round(step_bpp * P / ms_per_step / 1e6 / HBM_PEAK_GBPS, 4),
        "copy_kernel_gbps": round(copy_gbps, 1), "hbm_frac_of_copy_step": round(step_bpp * P / ms_per_step / 1e6 / copy_gbps, 4),
        "kernels": kernels, "dominant_kernel": dominant,
        "gate": {"norm": info.norm, "z": None if math.isnan(info.z) else info.z, "tripped": bool(info.tripped),
                 "live_step_norm": live_info.norm},
    }
    if fallback:
        res["fallback_step"] = fallback
    if args.diagnostics:
        d = B.gxpo_get_diagnostics(ctx)
        res["diagnostics"] = {k: getattr(d, k) for k, _ in d._fields_}
    cpu_inputs = None
    if want_cpu_inputs:
        # sampled only now, after every GPU measurement: large device-to-host copies ahead of
        # the timed region were seen to cost the following kernels a few percent
        S = min(args.cpu_sample, numels[0])
        cpu_inputs = {"theta": views["theta"][0][:S].cpu(), "g0": g0.tensors[0][:S].cpu(), "g1": g1.tensors[0][:S].cpu(),
                      "gs": gs.tensors[0][:S].cpu(), "S": S, "spec": spec, "cfg": cfg}
    # ---- release everything before the next workload ---------------------------------------------------------
    B.gxpo_destroy(ctx)
    del ctx, calls, g0, g1, gs, tensors, views, flat, gflat, quad, events, step_events, active_step
    gc.collect()
    torch.cuda.empty_cache()
    return res, cpu_inputs


def describe_layout(placement: dict, two_sets: bool) -> str:
    """The `hbm_layout` entry of the result: how the buffers were placed (layout.last_placement())."""
    if placement["kind"] == "ranked":
        text = "rank-aware placement (read streams of a slab in one DRAM rank" + (
            ", theta/m/v chunks chosen by measurement" if (placement["detail"] or {}).get("tuned") else "") + "), moments +32KiB mod 64KiB"
    elif placement["kind"] == "same-phase":
        text = "same-phase"
    else:
        text = "moments +32KiB mod 64KiB"
    if two_sets:
        text += "; two buffer sets, every pass reads one and writes the other (alternating state)"
    return text


def kernel_source_stamp() -> str:
    """Identifies the kernel source a hardware-counter figure was taken on."""
    with open(os.path.join(ROOT, "paper_2605_06755_amd", "csrc", "gxpo_kernels.hip"), "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:16]


def counter_traffic(kernel: str, workload: str):
    """HBM bytes per launch of `kernel` on `workload` from the committed rocprofv3 --pmc summary, if that summary was
    taken on the kernel source that is in the tree now; else None (the counters cannot be read from inside this run)."""
    tpath = os.path.join(ROOT, "profiles", f"traffic_{kernel}_{workload}.json")
    if not os.path.exists(tpath):
        return None, "no committed counter summary for this kernel and workload"
    try:
        rec = json.load(open(tpath))
    except Exception:
        return None, "counter summary unreadable"
    if rec.get("kernel_source_sha256_16") != kernel_source_stamp():
        return None, "the committed counter summary was taken on an older kernel source"
    return rec.get("hbm_bytes_per_launch"), f"profiles/{os.path.basename(tpath)} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, same kernel source)"


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (asked for --gpus {args.gpus}); "
              "sharding over data-parallel ranks is not implemented", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the GXPO engine has no CPU path", file=sys.stderr)
        sys.exit(2)
    from paper_2605_06755_amd import build as lib_build
    lib_build.ensure_built()                     # loads what is built; builds only if nothing is there
    torch.cuda.set_device(torch.device("cuda:0"))

    head_name = args.workload or HEADLINE
    head, cpu_inputs = measure(head_name, args, want_cpu_inputs=not args.no_cpu_baseline)
    others = {}
    if args.workload is None:
        for name in ALSO:
            try:
                others[name], _ = measure(name, args)
            except Exception as e:        # a workload that does not fit this box must not cost the headline its line
                others[name] = {"error": f"{type(e).__name__}: {e}"}
                gc.collect()
                torch.cuda.empty_cache()

    dominant = head["dominant_kernel"]
    dk = head["kernels"][dominant]
    traffic, traffic_source = counter_traffic(dominant, head_name)
    cpu_baseline = None
    if cpu_inputs is not None:
        cpu_baseline = time_oracle(cpu_inputs)

    out = {
        "metric": "GXPO active-step Gparams/s and achieved HBM GB/s (% of peak) on 1 MI355X",
        "value": head["gparams_per_s"],
        "unit": "Gparams/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "ms_per_step_median_events": head["ms_per_step_median_events"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": head["workload"], "params": head["params"], "tensors": head["tensors"],
                   "grad_dtype": head["grad_dtype"], "fused_step2": head["fused_step2"], "hbm_layout": head["hbm_layout"],
                   "bytes_per_param_per_step": head["bytes_per_param_per_step"]},
        "hbm_gbps_step": head["hbm_gbps_step"],
        "hbm_frac_of_peak_step": head["hbm_frac_of_peak_step"],
        "copy_kernel_gbps": head["copy_kernel_gbps"],
        "hbm_frac_of_copy_step": head["hbm_frac_of_copy_step"],
        "kernels": head["kernels"],
        "gate": head["gate"],
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": dk["gbps"], "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(dk["gbps"] / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "traffic_source": traffic_source, "timing": "median of per-launch HIP-event durations over the timed steps"},
        "cpu_baseline": cpu_baseline,
    }
    for k in ("fallback_step", "diagnostics"):
        if k in head:
            out[k] = head[k]
    if others:
        out["workloads"] = others
    print(json.dumps(out))


def time_oracle(inputs):
    """The fp64 oracle, as it stands, on the first S elements of the same
    buffers: one active step (five calls), repeated until ~10 s have passed."""
    import torch
    from oracle import gxpo_oracle as O
    spec, cfg, S = inputs["spec"], inputs["cfg"], inputs["S"]
    oc = O.GXPOConfig(
        optim=O.OptimConfig(spec["optimizer"], lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.adam_eps,
                            weight_decay=cfg.weight_decay),
        K=cfg.K, alpha=cfg.alpha, delta=cfg.delta, r_max=cfg.r_max,
        gate=O.GateConfig(tau=cfg.tau, window=cfg.window, eps=cfg.gate_eps))
    f = lambda t: t.to(dtype=torch.float64).numpy()
    orc = O.GXPOOracle(oc, [f(inputs["theta"])])
    g0, g1, gs = [f(inputs["g0"])], [f(inputs["g1"])], [f(inputs["gs"])]
    steps, t0 = 0, time.perf_counter()
    while True:
        orc.fast_step_1(g0)
        orc.fast_step_2(g1)
        orc.extrapolate(g0, g1)
        orc.slow_step(gs)
        orc.gate_step()
        steps += 1
        el = time.perf_counter() - t0
        if el >= 10.0 or steps >= 8:
            break
    out = {"value": round(S * steps / el / 1e9, 5), "unit": "Gparams/s", "cores": 1, "kind": "oracle",
           "sample": f"first {S} parameters of the same buffers, {steps} active step(s) of the fp64 C oracle "
                     f"(fast step x2, extrapolate, slow step + norm, gate), {el:.1f} s, single thread"}
    del orc

    # the same oracle, unchanged, on all host threads: each thread owns a contiguous range of the sample and
    # runs the calls on it; the per-range sums of squares are added in range order for the one gate step
    import threading
    T = max(1, min(16, len(os.sched_getaffinity(0))))
    if T > 1:
        cuts = [S * i // T for i in range(T + 1)]
        parts = [O.GXPOOracle(oc, [f(inputs["theta"][a:b])]) for a, b in zip(cuts, cuts[1:])]
        grads = [([g0[0][a:b]], [g1[0][a:b]], [gs[0][a:b]]) for a, b in zip(cuts, cuts[1:])]
        sums = [0.0] * T

        def work(i):
            o, (a0, a1, a_s) = parts[i], grads[i]
            o.fast_step_1(a0)
            o.fast_step_2(a1)
            o.extrapolate(a0, a1)
            o.slow_step(a_s)
            sums[i] = o.tensor_norms()[0] ** 2
        gate = O.RollingGate(oc.gate)
        steps_t, t0 = 0, time.perf_counter()
        while True:
            threads = [threading.Thread(target=work, args=(i,)) for i in range(T)]
            for th in threads:
                th.start()
            for th in threads:
                th.join()
            gate.step(steps_t, math.sqrt(math.fsum(sums)))
            steps_t += 1
            el_t = time.perf_counter() - t0
            if el_t >= 5.0 or steps_t >= 8:
                break
        out["all_threads"] = {"value": round(S * steps_t / el_t / 1e9, 5), "cores": T,
                              "note": f"{steps_t} step(s), {el_t:.1f} s; range split in the harness, oracle code unchanged"}
    return out


if __name__ == "__main__":
    main()
