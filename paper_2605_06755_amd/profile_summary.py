#!/usr/bin/env python3
"""Turns rocprofv3 CSV output of `bench.py --workload X` runs into the short summaries kept in profiles/.

Three runs of the same command feed one summary (rocprofv3 collects counters in runs of their own):

    rocprofv3 --kernel-trace --stats --output-format csv -d /tmp/gxpo_prof/prof_X      -- python3 /root/repo/bench.py --workload X --no-cpu-baseline --steps 10
    rocprofv3 --pmc FETCH_SIZE       --output-format csv -d /tmp/gxpo_prof/pmc_fetch_X -- python3 /root/repo/bench.py --workload X --no-cpu-baseline --steps 3 --warmup 1
    rocprofv3 --pmc WRITE_SIZE       --output-format csv -d /tmp/gxpo_prof/pmc_write_X -- python3 /root/repo/bench.py --workload X --no-cpu-baseline --steps 3 --warmup 1

    python3 -m paper_2605_06755_amd.profile_summary X /tmp/gxpo_prof/prof_X /tmp/gxpo_prof/pmc_fetch_X /tmp/gxpo_prof/pmc_write_X /tmp/gxpo_prof/prof_X.log

The last argument is the stdout of the kernel-trace run (bench.py's JSON line).  Writes
profiles/gxpo_kernels_<X>.md and profiles/traffic_<kernel>_<X>.json; the latter carries a hash of the
kernel source so that bench.py reports the counter figure only for the kernels it was measured on.

The counters are scaled by what they read for gxpo_stream_copy, the plain copy kernel of known size
that bench.py launches in the same run.
"""
from __future__ import annotations

import collections
import csv
import glob
import hashlib
import json
import os
import statistics
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def short(name: str) -> str:
    n = name.replace("void ", "").replace("gxpo::(anonymous namespace)::", "gxpo::")
    return n.split("(")[0]


def one(pattern: str) -> str:
    hits = sorted(glob.glob(pattern, recursive=True), key=os.path.getsize)
    if not hits:
        raise SystemExit(f"nothing matches {pattern}")
    return hits[-1]


def kernel_stats(d: str):
    rows = list(csv.DictReader(open(one(os.path.join(d, "**", "*_kernel_stats.csv")))))
    return [r for r in rows if "gxpo" in r["Name"]]


def full_size_durations(d: str):
    """kernel -> durations (ms) of its launches on the full grid (the largest grid the kernel was launched on);
    the placement probe's launches on small windows are left out."""
    per = collections.defaultdict(list)
    for r in csv.DictReader(open(one(os.path.join(d, "**", "*_kernel_trace.csv")))):
        if "gxpo" in r["Kernel_Name"]:
            per[short(r["Kernel_Name"])].append((int(r["Grid_Size_X"]), (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6))
    GRID.update({k: max(g for g, _ in v) for k, v in per.items()})
    return {k: [ms for g, ms in v if g == max(g for g, _ in v)] for k, v in per.items()}


GRID = {}          # kernel name -> largest grid it was launched on (tells the workload's kernels from the placement probe's)


def full_size_counter(d: str, counter: str):
    per = collections.defaultdict(list)
    for r in csv.DictReader(open(one(os.path.join(d, "**", "*_counter_collection.csv")))):
        if r["Counter_Name"] == counter and "gxpo" in r["Kernel_Name"]:
            per[short(r["Kernel_Name"])].append((int(r["Grid_Size"]), float(r["Counter_Value"])))
    GRID.update({k: max(g for g, _ in v) for k, v in per.items()})
    return {k: [x for g, x in v if g == max(g for g, _ in v)] for k, v in per.items()}


def kernel_of(call: str, names):
    """The kernel instantiation that serves `call` in this workload: of the matching names the one launched on the largest
    grid (the placement probe launches k_optim_step's fp32 instantiation on small windows whatever the workload's dtype)."""
    want = "k_fused_steps_extrapolate" if call.startswith("fused") else ("k_extrapolate" if call == "extrapolate" else "k_optim_step")
    hits = [n for n in names if want in n]
    return max(hits, key=lambda n: GRID.get(n, 0)) if hits else None


def main(argv):
    if len(argv) != 6:
        raise SystemExit(__doc__)
    tag, d_stats, d_fetch, d_write, bench_log = argv[1:]
    bench = json.loads([l for l in open(bench_log) if l.startswith("{")][-1])
    P = bench["config"]["params"]
    kern = dict(bench["kernels"])
    if "fallback_step" in bench:
        f = bench["fallback_step"]
        kern["fallback_step"] = {"ms": f["ms_per_step_median_events"], "bytes_per_param": f["bytes_per_param"], "gbps": f["gbps"],
                                 "frac_of_peak": f["frac_of_peak"]}
    n_copy = min(P, 1 << 30)
    out = [f"# rocprofv3 summary: GXPO engine kernels, workload `{tag}`\n",
           f"Workload: {bench['config']['workload']}; {P} parameters in {bench['config']['tensors']} tensor(s), "
           f"{bench['config']['grad_dtype']} gradients, HBM layout: {bench['config']['hbm_layout']}.\n",
           "## kernel trace (`--kernel-trace --stats`)\n",
           f"Command: `cd /tmp && TMPDIR=/tmp rocprofv3 --kernel-trace --stats --output-format csv -d /tmp/gxpo_prof/prof_{tag} -- "
           f"python3 /root/repo/bench.py --workload {tag} --no-cpu-baseline --steps {bench['steps']}`\n",
           "rocprofv3's own statistics, all launches of a kernel name together:\n",
           "| kernel | calls | avg ms | min ms | max ms | % of GPU time |", "|---|---|---|---|---|---|"]
    for r in kernel_stats(d_stats):
        out.append(f"| `{short(r['Name'])}` | {r['Calls']} | {float(r['AverageNs']) / 1e6:.4f} | {float(r['MinNs']) / 1e6:.4f} | "
                   f"{float(r['MaxNs']) / 1e6:.4f} | {r['Percentage']} |")
    out.append("\n`k_optim_step` serves several calls (probe pass, slow step, fallback step) and, in runs with the rank-aware "
               "allocator, the placement probe's thousands of launches on windows inside one 512 MiB chunk, which dominate its call count above. "
               "The same trace, launches on the full grid only, split by the call they belong to (nearest event-timed duration):\n")
    out.append("| call | kernel | launches | avg ms (rocprofv3 trace) | min | max | ms in bench.py (HIP events, median) | bytes/param | GB/s (trace avg) | % of 8 TB/s |")
    out.append("|---|---|---|---|---|---|---|---|---|---|")
    durs = full_size_durations(d_stats)
    for call, v in kern.items():
        kname = kernel_of(call, durs)
        if kname is None:
            continue
        same_kernel = [c for c in kern if kernel_of(c, durs) == kname]
        mine = [ms for ms in durs[kname] if min(same_kernel, key=lambda c: abs(kern[c]["ms"] - ms)) == call]
        if not mine:
            continue
        avg = sum(mine) / len(mine)
        gbps = v["bytes_per_param"] * P / avg / 1e6
        out.append(f"| {call} | `{kname}` | {len(mine)} | {avg:.4f} | {min(mine):.4f} | {max(mine):.4f} | {v['ms']} | {v['bytes_per_param']} | "
                   f"{gbps:.1f} | {gbps / 80:.1f} |")
    out.append(f"\nStep: {bench['ms_per_step']} ms wall-clock mean ({bench['ms_per_step_median_events']} ms median by events), "
               f"{bench['value']} Gparams/s, {bench['hbm_gbps_step']} GB/s algorithmic = {100 * bench['hbm_frac_of_peak_step']:.1f} % of peak; "
               f"plain copy kernel {bench['copy_kernel_gbps']} GB/s.")
    if "fallback_step" in bench:
        f = bench["fallback_step"]
        out.append(f"Fallback step: {f['ms_per_step']} ms, {f['gparams_per_s']} Gparams/s, {f['gbps']} GB/s = {100 * f['frac_of_peak']:.1f} % of peak.")
    out.append("")

    fetch, write = full_size_counter(d_fetch, "FETCH_SIZE"), full_size_counter(d_write, "WRITE_SIZE")
    copy_kib = n_copy * 4 / 1024
    cf, cw = max(fetch["gxpo::k_stream_copy"]), max(write["gxpo::k_stream_copy"])
    f_scale, w_scale = copy_kib / cf, copy_kib / cw
    out.append("## HBM traffic (`--pmc FETCH_SIZE`, then `--pmc WRITE_SIZE`, one run each)\n")
    out.append(f"Commands: `cd /tmp && rocprofv3 --pmc FETCH_SIZE --output-format csv -d /tmp/gxpo_prof/pmc_fetch_{tag} -- python3 /root/repo/bench.py --workload {tag} "
               f"--no-cpu-baseline --steps 3 --warmup 1`, the same with `WRITE_SIZE` into `/tmp/gxpo_prof/pmc_write_{tag}`, then "
               f"`cd /root/repo && python3 -m paper_2605_06755_amd.profile_summary {tag} /tmp/gxpo_prof/prof_{tag} /tmp/gxpo_prof/pmc_fetch_{tag} /tmp/gxpo_prof/pmc_write_{tag} "
               f"/tmp/gxpo_prof/prof_{tag}.log`.\n")
    out.append(f"Calibration: `gxpo::k_stream_copy` moves {n_copy} fp32 = {copy_kib:.0f} KiB each way per launch; the counters read "
               f"FETCH_SIZE = {cf:.0f} and WRITE_SIZE = {cw:.0f} for it, so FETCH_SIZE is scaled by {f_scale:.4f} and WRITE_SIZE by {w_scale:.4f}. "
               "Launches on the full grid only; a launch is attributed to the call whose read (write) bytes per parameter it is nearest to.\n")
    out.append("| call | kernel | FETCH_SIZE (raw, median) | WRITE_SIZE (raw, median) | HBM bytes / launch (scaled) | algorithmic bytes / launch | ratio |")
    out.append("|---|---|---|---|---|---|---|")
    g = 4 if bench["config"]["grad_dtype"] == "f32" else 2
    adam_in = 12                                                     # theta, m, v read by every pass of the AdamW workloads
    reads = {c: adam_in + (2 * g if c.startswith("fused") else g) for c in kern}
    traffic = {}
    for call, v in kern.items():
        kname = kernel_of(call, fetch)
        if kname is None or kname not in write or v["bytes_per_param"] == 0:
            continue
        rd, wr = reads[call], v["bytes_per_param"] - reads[call]
        same_kernel = [c for c in kern if kernel_of(c, fetch) == kname]
        fsel = [x for x in fetch[kname] if abs(x * f_scale * 1024 / P - rd) < 0.06 * rd]
        wsel = [x for x in write[kname]
                if min(same_kernel, key=lambda c: abs((kern[c]["bytes_per_param"] - reads[c]) - x * w_scale * 1024 / P)) == call
                and abs(x * w_scale * 1024 / P - wr) < 0.06 * wr + 0.05]
        if not fsel or not wsel:
            continue
        fm, wm = statistics.median(fsel), statistics.median(wsel)
        total = (fm * f_scale + wm * w_scale) * 1024
        alg = v["bytes_per_param"] * P
        out.append(f"| {call} | `{kname}` | {fm:.0f} | {wm:.0f} | {total:.4e} | {alg:.4e} | {total / alg:.4f} |")
        traffic[call] = (kname, round(total), alg)
    out.append("")
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    md = os.path.join(ROOT, "profiles", f"gxpo_kernels_{tag}.md")
    open(md, "w").write("\n".join(out))
    with open(os.path.join(ROOT, "paper_2605_06755_amd", "csrc", "gxpo_kernels.hip"), "rb") as fh:
        stamp = hashlib.sha256(fh.read()).hexdigest()[:16]
    for rname, (kname, total, alg) in traffic.items():
        json.dump({"kernel": kname, "call": rname, "workload": tag, "hbm_bytes_per_launch": total, "algorithmic_bytes_per_launch": alg,
                   "kernel_source_sha256_16": stamp, "source": f"profiles/gxpo_kernels_{tag}.md"},
                  open(os.path.join(ROOT, "profiles", f"traffic_{rname}_{tag}.json"), "w"), indent=1)
    print("\n".join(out))


if __name__ == "__main__":
    main(sys.argv)
