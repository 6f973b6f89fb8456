"""CPU-only checks of the library's host side: exported symbols, configuration
validation, the block plan for ragged tensor lists and the gate rule.  No
kernel is launched here."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

from oracle import gxpo_oracle as O
from paper_2605_06755_amd import binding as B
from paper_2605_06755_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "gxpo.h")).read()
    declared = set(re.findall(r"^\s*(?:int|void|const char \*)\s*\*?\s*(gxpo_\w+)\s*\(", header, flags=re.M))
    assert declared == set(B.EXPORTED_SYMBOLS), declared ^ set(B.EXPORTED_SYMBOLS)
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


@pytest.mark.parametrize("compiler,flags", [("gcc", ["-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror"]),
                                            ("g++", ["-std=c++11", "-Wall", "-Wextra", "-Werror"])])
def test_header_is_plain_c_and_cxx(compiler, flags, tmp_path):
    """The boundary is a C ABI: the header must compile on its own as strict C99 and as C++,
    and the struct sizes the binding assumes must be the compiler's."""
    import subprocess
    src = tmp_path / ("probe.c" if compiler == "gcc" else "probe.cpp")
    src.write_text('#include "gxpo.h"\n#include <stdio.h>\n'
                   'int main(void) { printf("%u %u %u %u %u %u\\n", (unsigned)sizeof(gxpo_tensor), (unsigned)sizeof(gxpo_config),\n'
                   '  (unsigned)sizeof(gxpo_gate_info), (unsigned)sizeof(gxpo_diagnostics), (unsigned)sizeof(gxpo_state),\n'
                   '  (unsigned)sizeof(gxpo_tensor_options)); return 0; }\n')
    exe = tmp_path / "probe"
    subprocess.check_call([compiler, *flags, "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    sizes = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    assert sizes == [ctypes.sizeof(t) for t in (B.gxpo_tensor, B.gxpo_config, B.gxpo_gate_info, B.gxpo_diagnostics,
                                                B.gxpo_state, B.gxpo_tensor_options)]


def test_plain_c_driver_links_against_the_library():
    """The gcc-built C99 program finds libgxpo.so and the HIP runtime; without a GPU it stops at its
    device check (exit status 2), with one it runs to the end (exit status 0)."""
    import subprocess
    from paper_2605_06755_amd import build as lib_build
    assert os.path.exists(lib_build.ABI_DRIVER), "run __graft_entry__.build() first"
    res = subprocess.run([lib_build.ABI_DRIVER], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert res.returncode in (0, 2), res.stdout


def test_struct_sizes_match_the_header_layout():
    # natural C layout of the header's structs on x86-64
    assert ctypes.sizeof(B.gxpo_tensor) == 8 + 7 * 8
    assert ctypes.sizeof(B.gxpo_config) == 12 * 4 + 11 * 8
    assert ctypes.sizeof(B.gxpo_tensor_options) == 2 * 8
    assert ctypes.sizeof(B.gxpo_diagnostics) == 9 * 8 + 8
    assert ctypes.sizeof(B.gxpo_gate_info) == 4 * 8 + 2 * 4 + 2 * 8
    assert ctypes.sizeof(B.gxpo_state) == 2 * 4 + 4 * 8 + 2 * 4 + 8 * B.GXPO_MAX_WINDOW


def test_default_config_is_valid():
    rc, msg = B.gxpo_validate_config(B.make_config())
    assert rc == B.GXPO_OK, msg


@pytest.mark.parametrize("kwargs,code", [
    (dict(K=1), B.GXPO_ERR_INVALID_ARG),
    (dict(K=0), B.GXPO_ERR_INVALID_ARG),
    (dict(K=4097), B.GXPO_ERR_INVALID_ARG),
    (dict(alpha=-0.1), B.GXPO_ERR_INVALID_ARG),
    (dict(alpha=1.5), B.GXPO_ERR_INVALID_ARG),
    (dict(alpha=float("nan")), B.GXPO_ERR_INVALID_ARG),
    (dict(lr=0.0), B.GXPO_ERR_INVALID_ARG),
    (dict(lr=-1e-3), B.GXPO_ERR_INVALID_ARG),
    (dict(delta=-1.0), B.GXPO_ERR_INVALID_ARG),
    (dict(r_max=0.0), B.GXPO_ERR_INVALID_ARG),
    (dict(window=1), B.GXPO_ERR_INVALID_ARG),
    (dict(window=B.GXPO_MAX_WINDOW + 1), B.GXPO_ERR_INVALID_ARG),
    (dict(gate_min_count=1), B.GXPO_ERR_INVALID_ARG),
    (dict(window=5, gate_min_count=6), B.GXPO_ERR_INVALID_ARG),
    (dict(gate_ddof=2), B.GXPO_ERR_INVALID_ARG),
    (dict(gate_eps=0.0), B.GXPO_ERR_INVALID_ARG),
    (dict(beta1=1.0), B.GXPO_ERR_INVALID_ARG),
    (dict(beta2=-0.1), B.GXPO_ERR_INVALID_ARG),
    (dict(copy_mask=8), B.GXPO_ERR_INVALID_ARG),
    (dict(diagnostics=2), B.GXPO_ERR_INVALID_ARG),
    (dict(explicit_steps=1), B.GXPO_ERR_INVALID_ARG),
    (dict(explicit_steps=3, diagnostics=1), B.GXPO_ERR_INVALID_ARG),
    (dict(clip_norm=-1.0), B.GXPO_ERR_INVALID_ARG),
    (dict(clip_norm=float("inf")), B.GXPO_ERR_INVALID_ARG),
    (dict(optimizer=7), B.GXPO_ERR_UNSUPPORTED),
    (dict(grad_dtype=2), B.GXPO_ERR_UNSUPPORTED),
])
def test_bad_configs_are_rejected_with_a_message(kwargs, code):
    rc, msg = B.gxpo_validate_config(B.make_config(**kwargs))
    assert rc == code
    assert msg


@pytest.mark.parametrize("kwargs", [dict(K=2), dict(K=4096), dict(alpha=0.0), dict(alpha=1.0), dict(delta=math.inf),
                                    dict(delta=0.0), dict(r_max=1.0), dict(optimizer="gd"), dict(grad_dtype="bf16"),
                                    dict(gate_min_count=2), dict(window=B.GXPO_MAX_WINDOW), dict(tau=-1.0), dict(explicit_steps=5),
                                    dict(clip_norm=1.0)])
def test_edge_configs_are_accepted(kwargs):
    rc, msg = B.gxpo_validate_config(B.make_config(**kwargs))
    assert rc == B.GXPO_OK, msg


def test_struct_size_mismatch_is_rejected():
    c = B.make_config()
    c.struct_size -= 4
    assert B.gxpo_validate_config(c)[0] == B.GXPO_ERR_INVALID_ARG


def test_init_rejects_bad_arguments_before_touching_the_gpu():
    out = ctypes.c_void_p()
    lib = B._lib
    cfg = B.make_config()
    assert lib.gxpo_init(ctypes.byref(out), ctypes.byref(cfg), None, 0) == B.GXPO_ERR_INVALID_ARG
    assert out.value is None and B.gxpo_last_error(None)
    t = (B.gxpo_tensor * 1)()
    t[0].numel = 16
    assert lib.gxpo_init(ctypes.byref(out), ctypes.byref(cfg), t, 1) == B.GXPO_ERR_INVALID_ARG      # theta NULL
    t[0].theta, t[0].theta_probe, t[0].m, t[0].v = 0x1004, 0x2000, 0x3000, 0x4000
    assert lib.gxpo_init(ctypes.byref(out), ctypes.byref(cfg), t, 1) == B.GXPO_ERR_ALIGNMENT
    assert "aligned" in B.gxpo_last_error(None)
    t[0].theta = 0x1000
    t[0].m = 0x1020                                                                                   # overlaps theta
    assert lib.gxpo_init(ctypes.byref(out), ctypes.byref(cfg), t, 1) == B.GXPO_ERR_INVALID_ARG
    assert "overlaps" in B.gxpo_last_error(None)
    t[0].m = None
    assert lib.gxpo_init(ctypes.byref(out), ctypes.byref(cfg), t, 1) == B.GXPO_ERR_INVALID_ARG      # AdamW needs m
    gd = B.make_config(optimizer="gd")
    t[0].m = 0x3000
    assert lib.gxpo_init(ctypes.byref(out), ctypes.byref(gd), t, 1) == B.GXPO_ERR_INVALID_ARG       # GD forbids m, v
    t[0].numel = 0
    assert lib.gxpo_init(ctypes.byref(out), ctypes.byref(cfg), t, 1) == B.GXPO_ERR_INVALID_ARG
    assert out.value is None


def test_layout_hint():
    assert B.gxpo_layout_hint(B.GXPO_BUF_THETA) == (0, 65536) and B.gxpo_layout_hint(B.GXPO_BUF_GRAD) == (0, 65536)
    assert B.gxpo_layout_hint(B.GXPO_BUF_M) == B.gxpo_layout_hint(B.GXPO_BUF_V) == (32768, 65536)
    with pytest.raises(B.GxpoError):
        B.gxpo_layout_hint(6)


# ---- block plan ---------------------------------------------------------------------------------
def test_block_plan_covers_every_element_exactly_once():
    rng = np.random.default_rng(0)
    numels = [1, 255, 256, 257, 4096, 1023, 5, 100000] + [int(x) for x in rng.integers(1, 50000, size=40)]
    start, epb = B.gxpo_plan_blocks(numels)
    assert epb == 256
    assert start[0] == 0 and len(start) == len(numels) + 1
    for t, n in enumerate(numels):
        nb = start[t + 1] - start[t]
        assert (nb - 1) * epb < n <= nb * epb


def test_block_plan_for_the_llama_layout():
    layout = synth.llama31_8b_layout()
    assert len(layout) == 290
    numels = [n for _, n in layout]
    assert sum(numels) == 8_030_257_152
    start, epb = B.gxpo_plan_blocks(numels)
    assert start[-1] == sum(-(-n // epb) for n in numels)
    assert start[-1] < 2 ** 31


def test_block_plan_rejects_too_large_and_empty():
    with pytest.raises(B.GxpoError):
        B.gxpo_plan_blocks([0])
    with pytest.raises(B.GxpoError):
        B.gxpo_plan_blocks([2 ** 40])


# ---- gate rule against the oracle's gate -----------------------------------------------------------
@pytest.mark.parametrize("window,min_count,ddof,tau", [(10, 0, 0, 3.0), (4, 2, 0, 1.0), (6, 3, 1, 2.0), (2, 0, 1, 0.5)])
def test_host_gate_matches_oracle_gate(window, min_count, ddof, tau):
    rng = np.random.default_rng(window * 7 + ddof)
    cfg = B.make_config(window=window, gate_min_count=min_count, gate_ddof=ddof, tau=tau, gate_eps=1e-8)
    for trial in range(20):
        st = B.new_state()
        orc = O.RollingGate(O.GateConfig(tau=tau, window=window, eps=1e-8, ddof=ddof,
                                         min_count=(min_count or None)))
        level = 1.0
        for t in range(40):
            if rng.random() < 0.05:
                level *= 3.0
            x = float(level * (1.0 + 0.01 * rng.normal()))
            info = B.gxpo_host_gate_step(cfg, st, x)
            ref = orc.step(t, x)
            assert bool(info.evaluated) == ref.evaluated
            assert info.t == t and st.t == t + 1
            if ref.evaluated:
                assert info.mu == pytest.approx(ref.mu, rel=1e-14)
                assert info.sigma == pytest.approx(ref.sigma, rel=1e-9, abs=1e-300)
                assert info.z == pytest.approx(ref.z, rel=1e-9, abs=1e-9)
            assert (info.s_star if info.s_star >= 0 else None) == ref.s_star
            assert list(st.window[:st.window_len]) == orc.buffer


def test_host_gate_at_the_largest_window():
    w = B.GXPO_MAX_WINDOW
    cfg = B.make_config(window=w, tau=5.0, gate_eps=1e-8)
    st = B.new_state()
    orc = O.RollingGate(O.GateConfig(tau=5.0, window=w, eps=1e-8))
    rng = np.random.default_rng(3)
    for t in range(2 * w + 50):
        x = float(10.0 + 0.1 * rng.normal() + (5.0 if t == 2 * w + 20 else 0.0))
        info = B.gxpo_host_gate_step(cfg, st, x)
        ref = orc.step(t, x)
        assert bool(info.evaluated) == ref.evaluated == (t >= w)
        assert (info.s_star if info.s_star >= 0 else None) == ref.s_star
        assert st.window_len == min(t + 1, w) and list(st.window[:st.window_len]) == orc.buffer
    assert st.s_star == 2 * w + 21


def test_host_gate_hand_case_and_nan():
    cfg = B.make_config(window=4, gate_min_count=2, tau=2.0, gate_eps=0.5)
    st = B.new_state()
    B.gxpo_host_gate_step(cfg, st, 1.0)
    B.gxpo_host_gate_step(cfg, st, 3.0)
    info = B.gxpo_host_gate_step(cfg, st, 5.0)               # mu 2, sigma 1, Z = 3 / 1.5 = 2 >= tau
    assert (info.mu, info.sigma, info.z, info.tripped, info.s_star) == (2.0, 1.0, 2.0, 1, 3)
    st = B.new_state()
    info = B.gxpo_host_gate_step(cfg, st, float("inf"))
    assert info.tripped == 1 and info.s_star == 1 and info.evaluated == 0


def test_gate_min_count_2_is_the_printed_algorithm_and_trips_on_an_early_spike():
    """Algorithm 1 evaluates the rule as soon as the buffer holds more than one norm.  With gate_min_count = 2 a
    spike at t = 2 (third step, two norms in the buffer) trips the gate: s* = 3 and, over T = 20 steps, 3 s* + (T - s*)
    backward passes.  With the default (the text's warm-up: evaluate once w norms are there) the same spike goes
    unseen and later steps judge against a buffer that holds it.  Oracle and library must agree on both readings."""
    norms = [1.00, 1.02, 5.00] + [1.0 + 0.01 * ((7 * i) % 5) for i in range(17)]
    T, w = len(norms), 10
    for min_count, want_s_star in ((2, 3), (0, None)):
        cfg = B.make_config(window=w, gate_min_count=min_count, tau=3.0, gate_eps=1e-8)
        st = B.new_state()
        orc = O.RollingGate(O.GateConfig(tau=3.0, window=w, eps=1e-8, min_count=(min_count or None)))
        passes = 0
        for t, x in enumerate(norms):
            active = st.s_star < 0 or st.t < st.s_star
            passes += 3 if active else 1
            if not active:
                st.t += 1                                    # what gxpo_fallback_step does to the step counter
                continue
            info = B.gxpo_host_gate_step(cfg, st, x)
            ref = orc.step(t, x)
            assert bool(info.evaluated) == ref.evaluated == (t >= (min_count or w))
            assert (info.s_star if info.s_star >= 0 else None) == ref.s_star
            if t == 2 and min_count == 2:
                assert info.tripped == 1 and info.z == pytest.approx((5.0 - 1.01) / (0.01 + 1e-8))
        assert (st.s_star if st.s_star >= 0 else None) == want_s_star
        s = want_s_star if want_s_star is not None else T
        assert passes == 3 * s + (T - s)


# ---- the product path fails loudly instead of falling back ------------------------------------------
def test_bench_refuses_more_than_one_gpu_and_a_missing_gpu():
    import subprocess
    import sys
    bench = os.path.join(ROOT, "bench.py")
    res = subprocess.run([sys.executable, bench, "--gpus", "2"], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=300)
    assert res.returncode != 0 and "one GPU" in res.stderr and not res.stdout.strip()
    import torch
    if not torch.cuda.is_available():
        res = subprocess.run([sys.executable, bench, "--steps", "1", "--warmup", "0"], stdout=subprocess.PIPE, stderr=subprocess.PIPE,
                             text=True, timeout=300)
        assert res.returncode != 0 and "no CPU path" in res.stderr and not res.stdout.strip()


def test_binding_import_fails_loudly_without_the_built_library(tmp_path):
    """A copy of the package without libgxpo.so must refuse to import its binding: there is no CPU fallback."""
    import shutil
    import subprocess
    import sys
    pkg = tmp_path / "paper_2605_06755_amd"
    pkg.mkdir()
    for name in ("__init__.py", "binding.py"):
        shutil.copy(os.path.join(ROOT, "paper_2605_06755_amd", name), pkg / name)
    res = subprocess.run([sys.executable, "-c", "import paper_2605_06755_amd.binding"], cwd=tmp_path, stdout=subprocess.PIPE,
                         stderr=subprocess.PIPE, text=True, timeout=300, env={**os.environ, "PYTHONPATH": str(tmp_path)})
    assert res.returncode != 0 and "ImportError" in res.stderr and "no CPU fallback" in res.stderr


def test_product_code_never_touches_the_oracle():
    """Only tests, the smoke check and bench.py's CPU-baseline leg may use oracle/."""
    for folder in ("paper_2605_06755_amd", "include"):
        for base, _, files in os.walk(os.path.join(ROOT, folder)):
            for f in files:
                if f.endswith((".py", ".h", ".hip", ".cpp", ".c")):
                    text = open(os.path.join(base, f)).read()
                    assert not re.search(r"^\s*(from|import)\s+oracle|gxpo_oracle", text, flags=re.M), f"{f} reaches into oracle/"
    bench = open(os.path.join(ROOT, "bench.py")).read()
    uses = [i for i, line in enumerate(bench.splitlines()) if "from oracle" in line or "import oracle" in line]
    start = bench.splitlines().index("def time_oracle(inputs):")
    assert uses and all(i > start for i in uses), "bench.py may import the oracle only inside its CPU-baseline leg"


# ---- rank-aware placement: the chunk plan (pure bookkeeping, no GPU) --------------------------------
def _plan_specs(numel, grad_itemsize=4, copy=True):
    specs = [dict(name=k, numel=numel, itemsize=4, group="read", phase_bytes=ph) for k, ph in (("theta", 0), ("m", 32768), ("v", 32768))]
    specs += [dict(name=f"g{i}", numel=numel, itemsize=grad_itemsize, group="read", phase_bytes=0) for i in range(3)]
    specs.append(dict(name="theta_probe", numel=numel, itemsize=4, group="write", phase_bytes=0))
    if copy:
        specs.append(dict(name="model_copy", numel=numel, itemsize=2, group="write", phase_bytes=0))
    return specs


@pytest.mark.parametrize("numel,grad_itemsize,copy", [(7_600_000_000, 4, True), (8_030_257_152, 2, False), (3_200_000_000, 4, False),
                                                       (300_000_004, 2, True)])
def test_chunk_plan_keeps_the_read_streams_of_a_slab_in_one_rank(numel, grad_itemsize, copy):
    from paper_2605_06755_amd import hbm_arena as A
    cb = A.CHUNK_BYTES
    specs = _plan_specs(numel, grad_itemsize, copy)
    need = sum(-(-(s["numel"] * s["itemsize"] + s["phase_bytes"]) // cb) for s in specs)
    # three ranks of 96 GiB, handed out the way a large allocation was seen to be: runs of chunks per rank, plus a few strays
    rng = np.random.default_rng(numel % 1000)
    labels = [0] * 128 + [1] * 192 + [2] * 64 + [0] * 64 + [2] * 100 + [3, 4]
    order = list(range(len(labels)))
    assert len(labels) >= need
    plan, slab_rank = A.plan_chunks(labels, specs, cb)
    used = [c for chunks in plan.values() for c in chunks]
    assert len(used) == len(set(used)) == need                            # every chunk at most once, every byte backed
    for s in specs:
        assert len(plan[s["name"]]) == -(-(s["numel"] * s["itemsize"] + s["phase_bytes"]) // cb)
    # per slab, all read buffers' chunks carry the slab's label (the pools are large enough here for that to hold throughout)
    for s in specs:
        per = max(1, A.SLAB_ELEMS * s["itemsize"] // cb)
        for k, c in enumerate(plan[s["name"]]):
            slab = k // per
            if s["group"] == "read":
                assert labels[c] == slab_rank[slab], (s["name"], k)
    # the write-only buffers avoid their slab's rank as long as another rank has chunks left
    wrong = sum(labels[c] == slab_rank[k // max(1, A.SLAB_ELEMS * s["itemsize"] // cb)]
                for s in specs if s["group"] == "write" for k, c in enumerate(plan[s["name"]]))
    assert wrong == 0
    # few changes of rank along the buffer: the planner stays in a rank while it has room
    assert sum(a != b for a, b in zip(slab_rank, slab_rank[1:])) <= 2
    # without scattering, chunks of a class are handed out in index order; with it, in a fixed other order over the same classes
    plain, plain_rank = A.plan_chunks(labels, specs, cb, scatter=False)
    assert plain_rank == slab_rank
    for s in specs:
        assert [labels[c] for c in plain[s["name"]]] == [labels[c] for c in plan[s["name"]]]
        by_label = {}
        for c in plain[s["name"]]:
            by_label.setdefault(labels[c], []).append(c)
        assert all(v == sorted(v) for v in by_label.values())
    again, _ = A.plan_chunks(labels, specs, cb)
    assert again == plan                                                   # the scattered order is a function of the labels alone
    assert any(plan[s["name"]] != plain[s["name"]] for s in specs)


def test_scatter_is_a_permutation():
    from paper_2605_06755_amd import hbm_arena as A
    for n in (0, 1, 2, 7, 192):
        for seed in (0, 1, 5):
            out = A._scatter(list(range(100, 100 + n)), seed)
            assert sorted(out) == list(range(100, 100 + n))
    assert A._scatter(list(range(192)), 0) != list(range(192))
    assert A._scatter(list(range(192)), 0) != A._scatter(list(range(192)), 1)
    # no regular stride survives: neighbours in the scattered order are rarely neighbours in memory
    out = A._scatter(list(range(192)), 2)
    assert sum(abs(a - b) == 1 for a, b in zip(out, out[1:])) < 12


def test_chunk_plan_spills_and_refuses():
    from paper_2605_06755_amd import hbm_arena as A
    cb = A.CHUNK_BYTES
    specs = _plan_specs((1 << 28) - (1 << 16), 4, copy=False)    # one slab: 2 chunks per fp32 buffer (phases included), 14 in all
    # no single class holds the 12 read chunks: the slab spills over classes instead of failing
    plan, slab_rank = A.plan_chunks([0] * 8 + [1] * 8, specs, cb)
    assert sum(len(v) for v in plan.values()) == 14 and len(slab_rank) == 1
    with pytest.raises(A.ArenaUnavailable):
        A.plan_chunks([0] * 13, specs, cb)
    # only the listed chunks may be used
    plan, _ = A.plan_chunks([0] * 40, specs, cb, available=list(range(20, 40)))
    assert min(c for v in plan.values() for c in v) >= 20


def test_choose_tuples_keeps_the_best_rated_candidate_and_never_reuses_a_chunk():
    from paper_2605_06755_amd import hbm_arena as A
    pools = {0: list(range(0, 40)), 1: list(range(100, 112))}
    positions = [0, 0, None, 1, 0, 1, 0]
    calls = []

    def rating(tup):
        return -float(sum((c % 7 - 3) ** 2 for c in tup))          # best: chunks with c % 7 == 3

    def measure(k, tup):
        calls.append((k, tup))
        assert len(set(tup)) == 3
        return rating(tup)

    tuples, seen = A.choose_tuples(pools, positions, 3, 8, measure, seed=3)
    assert tuples[2] is None and seen[2] == []
    flat = [c for t in tuples if t for c in t]
    assert len(flat) == len(set(flat)) == 18                       # no chunk twice
    for k, lab in enumerate(positions):
        if lab is not None:
            assert all(c in pools[lab] for c in tuples[k])
            rated = [rating(t) for kk, t in calls if kk == k]
            assert rating(tuples[k]) == max(rated) and 1 <= len(seen[k]) <= 8
    # a chunk chosen for one position is not offered to a later one
    for k, tup in list(calls):
        earlier = [c for kk in range(k) if tuples[kk] for c in tuples[kk]]
        assert not set(tup) & set(earlier)
    # same seed, same choice; pools are not modified
    again, _ = A.choose_tuples(pools, positions, 3, 8, measure, seed=3)
    assert again == tuples and pools[0] == list(range(0, 40))
    # the last position of a class can still be served when only its own chunks remain
    tuples, _ = A.choose_tuples({0: [5, 6, 7, 8, 9, 10]}, [0, 0], 3, 8, measure)
    assert sorted(c for t in tuples for c in t) == [5, 6, 7, 8, 9, 10]
    with pytest.raises(A.ArenaUnavailable):
        A.choose_tuples({0: [1, 2, 3, 4, 5]}, [0, 0], 3, 4, measure)


def test_chunk_plan_puts_the_second_buffer_set_into_another_rank():
    """Alternating state: theta, m, v and the first two gradient buffers (set 0) per slab in one rank, theta_probe,
    m_alt, v_alt and the last gradient buffer (set 1) together in another."""
    from paper_2605_06755_amd import hbm_arena as A
    cb = A.CHUNK_BYTES
    numel = 3_200_000_000
    f32 = lambda name, group, st, ph=0: dict(name=name, numel=numel, itemsize=4, group=group, set=st, phase_bytes=ph)
    specs = [f32("theta", "update", 0), f32("m", "update", 0, 32768), f32("v", "update", 0, 32768), f32("g0", "read", 0), f32("g1", "read", 0),
             f32("g2", "read", 1), f32("theta_probe", "update", 1), f32("m_alt", "update", 1, 32768), f32("v_alt", "update", 1, 32768),
             dict(name="model_copy", numel=numel, itemsize=2, group="write", phase_bytes=0)]
    labels = [0] * 190 + [1] * 188 + [2] * 170
    plan, rank0 = A.plan_chunks(labels, specs, cb)
    used = [c for v in plan.values() for c in v]
    assert len(used) == len(set(used))
    per = 2                                                                # chunks of an fp32 buffer per slab
    n_slabs = len(rank0)
    for slab in range(n_slabs):
        cls = {}
        for s in specs[:9]:
            chunks = plan[s["name"]][slab * per:(slab + 1) * per]
            labs = {labels[c] for c in chunks}
            assert len(labs) == 1, (s["name"], slab)
            cls.setdefault(s["set"], set()).update(labs)
        assert len(cls[0]) == 1 and len(cls[1]) == 1 and cls[0] != cls[1], slab   # each set together, the two apart
        assert cls[0] == {rank0[slab]}
    # with a single rank on offer the sets share it rather than fail
    plan, _ = A.plan_chunks([0] * 300, [dict(s, numel=1 << 28) for s in specs], cb)
    assert sum(len(v) for v in plan.values()) == 5 * 2 + 4 * 3 + 1         # 2^28 elements: 2 chunks per fp32 buffer, 3 with a phase, 1 for bf16


def test_bench_describes_the_placement_it_used():
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    ranked = {"kind": "ranked", "detail": {"tuned": {"positions": 12}}}
    assert bench.describe_layout(ranked, False).startswith("rank-aware placement") and "chosen by measurement" in bench.describe_layout(ranked, False)
    assert "chosen by measurement" not in bench.describe_layout({"kind": "ranked", "detail": {"tuned": None}}, False)
    assert bench.describe_layout({"kind": "phased", "detail": None}, False) == "moments +32KiB mod 64KiB"
    assert bench.describe_layout({"kind": "same-phase", "detail": None}, False) == "same-phase"
    both = bench.describe_layout(ranked, True)
    assert both.startswith("rank-aware placement") and both.endswith("(alternating state)")
    assert bench.describe_layout({"kind": "phased", "detail": None}, True).startswith("moments +32KiB")
