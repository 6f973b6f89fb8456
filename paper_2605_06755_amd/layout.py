"""Where the caller should put the engine's streams in HBM.

Every pass of the engine reads and writes several parameter-sized arrays at the
same element offset at the same time (theta, theta_probe, m, v and one or two
gradient buffers).  On MI355X the achieved bandwidth of such a pass depends on
how the base addresses of those arrays relate modulo 64 KiB: when all of them
share one phase the memory system serves them ~7 % slower than when about half
of the traffic sits 32 KiB out of phase with the other half (measured: 77 %
against 83.6 % of the 8 TB/s peak for the AdamW passes).

The rule used here: parameters, the probe buffer and gradients keep phase 0,
the AdamW moments m and v are placed 32 KiB (mod 64 KiB) away from them.  The
engine itself accepts any 16-byte aligned pointer; this module is allocation
plumbing for callers that want the fast layout.
"""
from __future__ import annotations

import sys

import torch

from . import binding as _B
from .hbm_arena import CHUNK_BYTES, ArenaUnavailable, RankedArena

# the library is the one place that states the placement
MOMENT_PHASE_BYTES, PHASE_PERIOD_BYTES = _B.gxpo_layout_hint(_B.GXPO_BUF_M)
assert _B.gxpo_layout_hint(_B.GXPO_BUF_THETA)[0] == 0 and _B.gxpo_layout_hint(_B.GXPO_BUF_GRAD)[0] == 0


def alloc_phased(numel: int, dtype, device, phase_bytes: int = 0, fill=None) -> torch.Tensor:
    """A contiguous 1-D tensor of `numel` elements whose first byte sits at
    `phase_bytes` modulo 64 KiB.  Over-allocates by at most 64 KiB."""
    es = torch.empty((), dtype=dtype).element_size()
    assert PHASE_PERIOD_BYTES % es == 0 and phase_bytes % es == 0
    slack = PHASE_PERIOD_BYTES // es
    raw = torch.empty(numel + slack, dtype=dtype, device=device)
    shift = (phase_bytes - raw.data_ptr()) % PHASE_PERIOD_BYTES
    out = raw[shift // es: shift // es + numel]
    assert out.data_ptr() % PHASE_PERIOD_BYTES == phase_bytes % PHASE_PERIOD_BYTES
    if fill is not None:
        out.fill_(fill)
    return out


RANKED_MIN_BYTES = 3 << 30          # below this a buffer is a single chunk: nothing to place
SPARE_CHUNKS_MIN = 96                # chunks taken beyond the need (at least; a third of the need if that is more): choice for the placement
CHUNKS_MIN = 240                     # ... and at least this many in all (120 GiB, more than one rank holds): the first 96 GiB a
                                     # process is given tend to lie in one rank, and theta_probe wants a rank of its own
TUNE_CANDIDATES = 16                # candidate (theta, m, v) chunk triples timed per chunk position
_last_placement = {"kind": None, "detail": None}


def last_placement() -> dict:
    """{'kind': 'ranked' | 'phased' | 'arena', 'detail': ...} of the most recent alloc_engine_state call."""
    return dict(_last_placement)


def alloc_engine_state(numel: int, device, *, adam: bool = True, model_copy: bool = False, grad_dtype=torch.float32,
                       n_grad_buffers: int = 3, arena: bool = False, phases_kib=None, placement: str = "auto",
                       with_probe: bool = True, probe_is_read: bool = False, alternating: bool = False, verbose: bool = False):
    """Flat buffers for one engine context in the fast layout: a dict with
    theta, theta_probe, (m, v), (m_alt, v_alt), (model_copy) and a list of gradient buffers.

    alternating: also allocate m_alt, v_alt, the second buffers for the moments;
    the engine then reads one of the sets {theta, m, v} / {theta_probe, m_alt,
    v_alt} and writes the other in every pass that advances the state.  The
    rank-aware placement puts the two sets into different DRAM ranks, the
    first two gradient buffers next to the first set and the third (the
    slow step's) next to the second.

    placement: "ranked" = rank-aware placement through HIP's virtual-memory API
    (hbm_arena.py: chunks of a rank handed out in scattered order, the chunks of
    theta, m, v then chosen by measurement; "ranked-scatter" = without that
    choice, "ranked-adjacent" = chunks in index order, both for comparison); "phased" = one plain allocation per buffer with the 64 KiB
    phase rule only; "auto" = ranked for workloads of 3 GiB and more where the
    API is available, phased otherwise.  `last_placement()` tells which one
    the most recent call used.
    `probe_is_read`: the schedule reads theta_probe back (unfused second fast
    step, explicit lookahead), so it is placed with the read streams; with
    the fused schedule the engine only ever writes it.
    `phases_kib` overrides the phases for experiments: a dict name -> KiB
    (names theta, theta_probe, m, v, model_copy, g0, g1, g2)."""
    if alternating and not (adam and with_probe) or alternating and arena:
        raise ValueError("alternating state needs AdamW and theta_probe (and is not offered with arena=True)")
    if arena:
        _last_placement.update(kind="arena", detail=None)
        return _alloc_arena(numel, device, adam, model_copy, grad_dtype, n_grad_buffers)
    _last_placement.update(kind="phased", detail=None)
    if placement not in ("auto", "ranked", "ranked-scatter", "ranked-adjacent", "phased"):
        raise ValueError(placement)
    if placement != "phased":
        gs = torch.empty((), dtype=grad_dtype).element_size()
        total = numel * (4 * (1 + int(with_probe) + 2 * int(adam) + 2 * int(alternating)) + 2 * int(model_copy) + gs * n_grad_buffers)
        if placement.startswith("ranked") or total >= RANKED_MIN_BYTES:
            try:
                return _alloc_ranked(numel, device, adam, model_copy, grad_dtype, n_grad_buffers, phases_kib, with_probe,
                                     probe_is_read, verbose, scatter=placement != "ranked-adjacent",
                                     tune=TUNE_CANDIDATES if placement in ("auto", "ranked") else 0, alternating=alternating)
            except Exception as e:          # the virtual-memory API refused, or the placement probe failed
                if placement.startswith("ranked"):
                    raise
                print(f"[layout] rank-aware placement not available ({type(e).__name__}: {e}); using plain phased allocations",
                      file=sys.stderr)
                torch.cuda.empty_cache()
    ph = _default_phases_kib(grad_dtype)
    ph.update(phases_kib or {})
    out = {"theta": alloc_phased(numel, torch.float32, device, int(ph["theta"] * 1024)),
           "theta_probe": alloc_phased(numel, torch.float32, device, int(ph["theta_probe"] * 1024))}
    if adam:
        out["m"] = alloc_phased(numel, torch.float32, device, int(ph["m"] * 1024), fill=0.0)
        out["v"] = alloc_phased(numel, torch.float32, device, int(ph["v"] * 1024), fill=0.0)
    if alternating:
        out["m_alt"] = alloc_phased(numel, torch.float32, device, int(ph["m"] * 1024), fill=0.0)
        out["v_alt"] = alloc_phased(numel, torch.float32, device, int(ph["v"] * 1024), fill=0.0)
    if model_copy:
        out["model_copy"] = alloc_phased(numel, torch.bfloat16, device, int(ph["model_copy"] * 1024))
    grads = [alloc_phased(numel, grad_dtype, device, int(ph.get(f"g{i}", 0) * 1024)) for i in range(n_grad_buffers)]
    if not with_probe:
        del out["theta_probe"]
    return out, grads


def _default_phases_kib(grad_dtype) -> dict:
    """Base address modulo 64 KiB, in KiB, of every buffer: the moments half a period away from the rest.  Two bf16
    gradient streams read side by side (the fused pass) do slightly better 1 KiB apart: measured +0.6 % on that pass."""
    ph = {"theta": 0, "theta_probe": 0, "m": MOMENT_PHASE_BYTES // 1024, "v": MOMENT_PHASE_BYTES // 1024, "model_copy": 0}
    if grad_dtype == torch.bfloat16:
        ph["g1"] = 1
    return ph


def _alloc_ranked(numel, device, adam, model_copy, grad_dtype, n_grad_buffers, phases_kib, with_probe, probe_is_read, verbose,
                  scatter=True, tune=0, alternating=False):
    """All buffers from one RankedArena: slab by slab, theta, m, v and the gradients share a rank;
    theta_probe and the bf16 copy (only ever written by the engine) come from another.  With alternating
    state the second set (theta_probe, m_alt, v_alt) and the last gradient buffer, which the slow step reads
    next to it, share that other rank."""
    ph = _default_phases_kib(grad_dtype)
    ph.update(phases_kib or {})
    specs = [dict(name="theta", numel=numel, dtype=torch.float32, group="update", phase_bytes=int(ph["theta"] * 1024))]
    if adam:
        specs += [dict(name=k, numel=numel, dtype=torch.float32, group="update", phase_bytes=int(ph[k] * 1024)) for k in ("m", "v")]
    specs += [dict(name=f"g{i}", numel=numel, dtype=grad_dtype, group="read", phase_bytes=int(ph.get(f"g{i}", 0) * 1024),
                   set=1 if alternating and i == n_grad_buffers - 1 and n_grad_buffers > 1 else 0)
              for i in range(n_grad_buffers)]
    if alternating:
        specs += [dict(name=k, numel=numel, dtype=torch.float32, group="update", set=1, phase_bytes=int(ph[p] * 1024))
                  for k, p in (("theta_probe", "theta_probe"), ("m_alt", "m"), ("v_alt", "v"))]
    elif with_probe:
        specs.append(dict(name="theta_probe", numel=numel, dtype=torch.float32, group="read" if probe_is_read else "write",
                          phase_bytes=int(ph["theta_probe"] * 1024)))
    if model_copy:
        specs.append(dict(name="model_copy", numel=numel, dtype=torch.bfloat16, group="write", phase_bytes=int(ph["model_copy"] * 1024)))
    cb = CHUNK_BYTES
    need = sum(-(-(s["numel"] * torch.empty((), dtype=s["dtype"]).element_size() + s["phase_bytes"]) // cb) for s in specs)
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info(device)
    # spare chunks give the placement a choice of ranks; leave room for the caller's temporaries
    budget = (free - (12 << 30)) // cb
    if budget < need:
        raise ArenaUnavailable(f"{need} chunks needed, room for {budget}")
    n_chunks = int(min(budget, max(CHUNKS_MIN, need + max(SPARE_CHUNKS_MIN, need // 3))))
    ar = RankedArena(device, n_chunks)
    try:
        labels = ar.classify(verbose=verbose)
        bufs = ar.build(specs, scatter=scatter, tune=tune, verbose=verbose)
    except Exception:
        ar.close()
        raise
    if verbose:
        counts = {lab: labels.count(lab) for lab in sorted(set(labels))}
        print(f"[layout] {n_chunks} chunks of {cb >> 20} MiB in ranks {counts}; read streams per slab in ranks {ar.slab_rank}", file=sys.stderr)
    counts = {lab: labels.count(lab) for lab in sorted(set(labels))}
    _last_placement.update(kind="ranked", detail={"chunk_mib": cb >> 20, "chunks_per_rank": counts, "slab_rank": list(ar.slab_rank),
                                                   "order": "scattered" if scatter else "index", "tuned": ar.tuned,
                                                   "alternating": bool(alternating)})
    out = {k: bufs[k] for k in ("theta", "theta_probe", "m", "v", "m_alt", "v_alt", "model_copy") if k in bufs}
    for k in ("m", "v", "m_alt", "v_alt"):
        if k in out:
            out[k].zero_()
    grads = [bufs[f"g{i}"] for i in range(n_grad_buffers)]
    return out, grads


def _alloc_arena(numel, device, adam, model_copy, grad_dtype, n_grad_buffers):
    """Everything carved from ONE allocation at a 2 MiB-multiple pitch."""
    two_mb = 2 << 20
    pitch = -(-(numel * 4) // two_mb) * two_mb + two_mb
    names = ["theta", "theta_probe"] + (["m", "v"] if adam else []) + (["model_copy"] if model_copy else [])
    n_arr = len(names) + n_grad_buffers
    raw = torch.empty(pitch * n_arr + two_mb, dtype=torch.uint8, device=device)
    start = (-raw.data_ptr()) % two_mb
    out, grads = {}, []
    for k in range(n_arr):
        name = names[k] if k < len(names) else None
        phase = MOMENT_PHASE_BYTES if name in ("m", "v") else 0
        dt = torch.float32 if name in ("theta", "theta_probe", "m", "v") else (torch.bfloat16 if name == "model_copy" else grad_dtype)
        es = torch.empty((), dtype=dt).element_size()
        lo = start + k * pitch + phase
        t = raw[lo: lo + numel * es].view(dt)
        if name in ("m", "v"):
            t.zero_()
        if name:
            out[name] = t
        else:
            grads.append(t)
    return out, grads
