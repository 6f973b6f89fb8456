"""Rank-aware placement of the engine's buffers in MI355X's HBM.

What was measured on this part (profiles/hbm_rank_placement.md): the 288 GiB of
HBM3E behave as three regions of 96 GiB of physical memory -- the three ranks of
the 12-high stacks.  A pass that reads several streams at the same element
offset runs ~4 % slower when one of its read streams lies in another rank than
the rest (every switch between ranks on a channel costs bus time), while a
stream that is only written is best kept in a rank the pass does not read.  A
plain allocation of tens of GiB is backed by power-of-two physical blocks that
land in whichever rank has room, so with parameter-sized buffers of 6-30 GiB
the streams of a pass end up in different ranks by accident: that is the "large
buffers lose 3 %" effect.

This module is allocation plumbing that removes the accident.  It takes
physical memory in chunks through HIP's virtual-memory API (hipMemCreate),
finds out by timing which chunks share a rank (the engine's own fallback step
is the probe: parameters and moments in a reference chunk, the gradient in the
candidate), and then maps the chunks into one contiguous address range per
buffer so that, slab by slab, the streams a pass reads together sit in the same
rank and the write-only streams (theta_probe, the bf16 model copy) in another.
Inside a rank the chunks are handed out in a scattered order, and the chunks
of the three streams that are read and written -- theta, m, v -- are chosen
per 512 MiB position by timing candidate triples with the same probe: which
chunks meet there moves the pass by several percent, with no pattern in the
chunk numbers to plan by.
Every buffer stays an ordinary contiguous device array; the engine sees plain
pointers and knows nothing of this.
"""
from __future__ import annotations

import ctypes
import sys
from typing import Dict, List, Optional, Sequence

import torch

from . import binding as _B

CHUNK_BYTES = 512 << 20
SLAB_ELEMS = 1 << 28              # co-location unit: 2 chunks of an fp32 buffer, 1 chunk of a bf16 buffer
_HIP_MEM_ALLOCATION_TYPE_PINNED = 1
_HIP_MEM_LOCATION_TYPE_DEVICE = 1
_HIP_MEM_ACCESS_READ_WRITE = 3


class _Loc(ctypes.Structure):
    _fields_ = [("type", ctypes.c_int), ("id", ctypes.c_int)]


class _AllocFlags(ctypes.Structure):
    _fields_ = [("compressionType", ctypes.c_ubyte), ("gpuDirectRDMACapable", ctypes.c_ubyte), ("usage", ctypes.c_ushort)]


class _Prop(ctypes.Structure):
    _fields_ = [("type", ctypes.c_int), ("requestedHandleType", ctypes.c_int), ("location", _Loc),
                ("win32HandleMetaData", ctypes.c_void_p), ("allocFlags", _AllocFlags)]


class _Access(ctypes.Structure):
    _fields_ = [("location", _Loc), ("flags", ctypes.c_int)]


class ArenaUnavailable(RuntimeError):
    """The virtual-memory API is missing or refused a call; callers fall back to plain allocations."""


_hip = None


def _runtime():
    global _hip
    if _hip is None:
        try:
            _hip = ctypes.CDLL("libamdhip64.so")
            _hip.hipGetErrorString.restype = ctypes.c_char_p
            for name in ("hipMemCreate", "hipMemAddressReserve", "hipMemMap", "hipMemSetAccess", "hipMemUnmap", "hipMemRelease",
                         "hipMemAddressFree"):
                getattr(_hip, name)
        except (OSError, AttributeError) as e:
            raise ArenaUnavailable(f"HIP virtual-memory API not available: {e}")
    return _hip


def _ck(rc: int, what: str):
    if rc != 0:
        raise ArenaUnavailable(f"{what} failed: {_runtime().hipGetErrorString(rc).decode()} ({rc})")


class _View:
    """What torch wraps: a typed window of mapped device memory that keeps its arena alive."""

    def __init__(self, arena, ptr: int, numel: int, typestr: str):
        self._arena = arena
        self.__cuda_array_interface__ = {"shape": (numel,), "typestr": typestr, "data": (ptr, False), "version": 3, "strides": None}


_TYPESTR = {torch.float32: "<f4", torch.uint8: "|u1", torch.int16: "<i2"}


def _scatter(chunks: List[int], seed: int) -> List[int]:
    """A fixed pseudo-random order of `chunks` (Fisher-Yates driven by a 64-bit LCG): the same plan for the same labels."""
    out, x = list(chunks), (seed * 0x9E3779B97F4A7C15 + 0xD1B54A32D192ED03) & (2 ** 64 - 1)
    for i in range(len(out) - 1, 0, -1):
        x = (x * 6364136223846793005 + 1442695040888963407) & (2 ** 64 - 1)
        j = (x >> 33) % (i + 1)
        out[i], out[j] = out[j], out[i]
    return out


def plan_chunks(labels: Sequence[int], specs: Sequence[dict], chunk_bytes: int = CHUNK_BYTES, available: Optional[Sequence[int]] = None,
                scatter: bool = True):
    """Which chunk backs which part of which buffer.  Pure bookkeeping (no GPU): `labels[i]` is the rank class of chunk
    i, `specs` are dicts with name, numel, itemsize, group ('update' = read and written, 'read', or 'write'),
    optionally set (0 or 1, default 0) and phase_bytes; all buffers index the same elements.  Per slab of SLAB_ELEMS
    elements the chunks of every 'update' and 'read' buffer of set 0 come from one class (the planner stays in a class
    while it has room for a whole slab, then moves to the class with most room), those of set 1 -- the second buffer
    set of the alternating schedule, which a pass writes while it reads set 0, and the other way round -- from one
    other class; 'write' buffers are served afterwards from what is left, away from set 0's class where possible.
    Inside a class the chunks are handed out in a fixed pseudo-random order (`scatter`) rather than in index order:
    streams that advance in step through neighbouring or evenly spaced chunks of physical memory were measured
    0.5-1.5 % slower than streams whose chunks have no regular relation to each other.
    Returns (name -> chunk ids in address order, class of set 0 for each slab)."""
    free: Dict[int, List[int]] = {}
    for i in (range(len(labels)) if available is None else available):
        free.setdefault(labels[i], []).append(i)
    for lab in free:
        free[lab] = _scatter(sorted(free[lab]), lab) if scatter else sorted(free[lab])
    per_slab = {s["name"]: max(1, SLAB_ELEMS * s["itemsize"] // chunk_bytes) for s in specs}
    need = {s["name"]: -(-(s["numel"] * s["itemsize"] + s.get("phase_bytes", 0)) // chunk_bytes) for s in specs}
    n_slabs = max(-(-need[s["name"]] // per_slab[s["name"]]) for s in specs)
    plan = {s["name"]: [] for s in specs}
    wants = lambda s, slab: max(0, min(per_slab[s["name"]], need[s["name"]] - slab * per_slab[s["name"]]))
    together = [[s for s in specs if s["group"] in ("read", "update") and s.get("set", 0) == k] for k in (0, 1)]
    writes = [s for s in specs if s["group"] == "write"]

    # 1. which class hosts each set's streams of each slab: stay while a whole slab fits, then move to the roomiest
    #    class; set 1 takes a class other than set 0's as long as one has room
    left = {lab: len(lst) for lab, lst in free.items()}
    roomiest = lambda: sorted(left, key=lambda lab: (-left[lab], lab))
    slab_rank = [[], []]
    current = [None, None]
    for slab in range(n_slabs):
        for k in (0, 1):
            want = sum(wants(s, slab) for s in together[k])
            if not together[k]:
                slab_rank[k].append(None)
                continue
            avoid = slab_rank[0][slab] if k == 1 else None
            if current[k] is None or left[current[k]] < want or current[k] == avoid:
                fits = [lab for lab in roomiest() if left[lab] >= want]
                fits = [lab for lab in fits if lab != avoid] or fits
                current[k] = fits[0] if fits else None
            slab_rank[k].append(current[k])                # None: no class can hold this set's streams of the slab whole
            if current[k] is not None:
                left[current[k]] -= want

    def take(label_order, count):
        out = []
        for lab in label_order:
            while free.get(lab) and len(out) < count:
                out.append(free[lab].pop(0))
            if len(out) == count:
                break
        if len(out) < count:
            raise ArenaUnavailable("not enough chunks for the requested buffers")
        return out

    room = lambda: sorted(free, key=lambda lab: (-len(free[lab]), lab))
    # 2. the co-located streams, slab by slab, from their class; slabs no class could hold whole spill over classes
    for k in (0, 1):
        for slab in range(n_slabs):
            if slab_rank[k][slab] is not None:
                for s in together[k]:
                    plan[s["name"]] += [(slab, c) for c in take([slab_rank[k][slab]], wants(s, slab))]
    for k in (0, 1):
        for slab in range(n_slabs):
            if together[k] and slab_rank[k][slab] is None:
                slab_rank[k][slab] = room()[0]
                for s in together[k]:
                    if wants(s, slab):
                        plan[s["name"]] += [(slab, c) for c in take(room(), wants(s, slab))]
    # 3. the write-only streams, from what is left, away from the class their slab is read from
    for slab in range(n_slabs):
        order = [lab for lab in room() if lab != slab_rank[0][slab]] + [slab_rank[0][slab]]
        for s in writes:
            if wants(s, slab):
                plan[s["name"]] += [(slab, c) for c in take(order, wants(s, slab))]
    return {name: [c for _, c in sorted(v, key=lambda x: x[0])] for name, v in plan.items()}, slab_rank[0]


def _lcg(seed: int):
    x = (seed * 0x9E3779B97F4A7C15 + 0xD1B54A32D192ED03) & (2 ** 64 - 1)
    while True:
        x = (x * 6364136223846793005 + 1442695040888963407) & (2 ** 64 - 1)
        yield x >> 33


def choose_tuples(pools: Dict[int, List[int]], positions: Sequence[Optional[int]], width: int, candidates: int, measure, seed: int = 0):
    """Best-of-several choice of chunk tuples, one tuple per position.  Pure bookkeeping around `measure`:
    `positions[k]` is the class position k draws from (None: leave it alone), `pools[class]` the chunks it may use.
    For every position up to `candidates` tuples of `width` distinct chunks are drawn from what is left of the pool,
    `measure(k, tuple)` rates each (higher is better), the best is kept and its chunks leave the pool.  A pool that
    runs short of `width` chunks is an error: the caller sizes the pools so that every position can be served.
    Returns (tuples, one per position or None; ratings seen per position)."""
    rnd = _lcg(seed)
    left = {lab: list(v) for lab, v in pools.items()}
    still = {lab: sum(1 for p in positions if p == lab) for lab in left}          # positions yet to serve per class
    out, seen = [], []
    for k, lab in enumerate(positions):
        if lab is None:
            out.append(None)
            seen.append([])
            continue
        pool = left[lab]
        if len(pool) < width * still[lab]:
            raise ArenaUnavailable("pool too small for the positions that draw from it")
        n_cand = candidates if len(pool) > width else 1
        best, ratings, tried = None, [], set()
        for _ in range(n_cand):
            idx = list(range(len(pool)))
            for i in range(width):                                                 # partial Fisher-Yates
                j = i + next(rnd) % (len(idx) - i)
                idx[i], idx[j] = idx[j], idx[i]
            tup = tuple(pool[i] for i in idx[:width])
            if tup in tried:
                continue
            tried.add(tup)
            r = measure(k, tup)
            ratings.append(r)
            if best is None or r > best[0]:
                best = (r, tup)
        out.append(best[1])
        seen.append(ratings)
        for c in best[1]:
            pool.remove(c)
        still[lab] -= 1
    return out, seen


class RankedArena:
    """Physical chunks of one GPU's HBM, labelled by rank, and the buffers mapped from them."""

    def __init__(self, device: torch.device, n_chunks: int, chunk_bytes: int = CHUNK_BYTES):
        hip = _runtime()
        self.device = torch.device(device)
        self.dev_index = self.device.index if self.device.index is not None else torch.cuda.current_device()
        self.chunk_bytes = chunk_bytes
        self.handles: List[Optional[ctypes.c_void_p]] = []
        self.labels: List[int] = []
        self._ranges = []                        # (va, bytes) reserved
        self._mapped = []                        # (va, bytes) mapped, one per chunk
        self._closed = False
        prop = _Prop()
        prop.type = _HIP_MEM_ALLOCATION_TYPE_PINNED
        prop.location = _Loc(_HIP_MEM_LOCATION_TYPE_DEVICE, self.dev_index)
        self._access = _Access(_Loc(_HIP_MEM_LOCATION_TYPE_DEVICE, self.dev_index), _HIP_MEM_ACCESS_READ_WRITE)
        try:
            for _ in range(n_chunks):
                h = ctypes.c_void_p()
                _ck(hip.hipMemCreate(ctypes.byref(h), ctypes.c_size_t(chunk_bytes), ctypes.byref(prop), ctypes.c_ulonglong(0)), "hipMemCreate")
                self.handles.append(h)
        except ArenaUnavailable:
            self.close()
            raise

    # ---- address ranges ------------------------------------------------------------------------
    def _reserve(self, nbytes: int) -> int:
        va = ctypes.c_void_p()
        _ck(_runtime().hipMemAddressReserve(ctypes.byref(va), ctypes.c_size_t(nbytes), ctypes.c_size_t(2 << 20), None, ctypes.c_ulonglong(0)),
            "hipMemAddressReserve")
        self._ranges.append((va.value, nbytes))
        return va.value

    def _map(self, va: int, chunk: int):
        hip = _runtime()
        _ck(hip.hipMemMap(ctypes.c_void_p(va), ctypes.c_size_t(self.chunk_bytes), ctypes.c_size_t(0), self.handles[chunk], ctypes.c_ulonglong(0)), "hipMemMap")
        self._mapped.append((va, self.chunk_bytes))
        _ck(hip.hipMemSetAccess(ctypes.c_void_p(va), ctypes.c_size_t(self.chunk_bytes), ctypes.byref(self._access), ctypes.c_size_t(1)), "hipMemSetAccess")

    def _unmap_all(self):
        hip = _runtime()
        for va, nbytes in self._mapped:
            hip.hipMemUnmap(ctypes.c_void_p(va), ctypes.c_size_t(nbytes))
        self._mapped = []
        for va, nbytes in self._ranges:
            hip.hipMemAddressFree(ctypes.c_void_p(va), ctypes.c_size_t(nbytes))
        self._ranges = []

    def _tensor(self, ptr: int, numel: int, dtype) -> torch.Tensor:
        if dtype == torch.bfloat16:          # the array interface has no bf16: wrap as int16, reinterpret
            return torch.as_tensor(_View(self, ptr, numel, "<i2"), device=self.device).view(torch.bfloat16)
        return torch.as_tensor(_View(self, ptr, numel, _TYPESTR[dtype]), device=self.device)

    # ---- which chunks share a rank ----------------------------------------------------------------
    def classify(self, verbose: bool = False) -> List[int]:
        """Labels every chunk with a class id such that chunks of one class behave as one rank: the
        engine's fallback step (reads theta, m, v, g; writes theta, m, v) is timed with theta, m, v in a
        reference chunk and g in each candidate; candidates in the reference's rank run measurably
        faster.  Repeats with a new reference among the chunks still unlabelled."""
        n = len(self.handles)
        cb = self.chunk_bytes
        va = self._reserve(n * cb)
        for i in range(n):
            self._map(va + i * cb, i)
        E = cb // 16                                       # four fp32 windows per chunk
        win = lambda chunk, k: self._tensor(va + chunk * cb + k * E * 4 + (32768 if k in (1, 2) else 0), E - 16384, torch.float32)
        cfg = _B.make_config(K=2, lr=1e-9, weight_decay=0.0, delta=0.0)
        labels = [-1] * n
        next_label = 0
        todo = list(range(n))
        grads = {}

        def measure(ctx, c, launches):
            if c not in grads:
                grads[c] = win(c, 3)
                grads[c].normal_(std=0.05)
            g = grads[c]
            _B.gxpo_fallback_step(ctx, [g])
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(launches):
                _B.gxpo_fallback_step(ctx, [g])
            b.record()
            b.synchronize()
            return launches * 28.0 * g.numel() / a.elapsed_time(b) / 1e6

        while todo and next_label < 6:
            ref = todo[0]
            th, m, v = win(ref, 0), win(ref, 1), win(ref, 2)
            th.normal_(std=0.02)
            m.zero_()
            v.fill_(1e-4)
            ctx = _B.gxpo_init(cfg, [dict(theta=th, m=m, v=v)])
            st = _B.gxpo_get_state(ctx)
            st.s_star = 0
            _B.gxpo_set_state(ctx, st)
            # disturbances only ever make a measurement slower, so the best of several counts
            rate = {c: max(measure(ctx, c, 4), measure(ctx, c, 4)) for c in todo}
            lo_c, hi_c = min(rate.values()), max(rate.values())
            for _ in range(8):                              # two-means on a line
                cut = (lo_c + hi_c) / 2
                lows = [r for r in rate.values() if r <= cut]
                highs = [r for r in rate.values() if r > cut]
                if not lows or not highs:
                    break
                lo_c, hi_c = sum(lows) / len(lows), sum(highs) / len(highs)
            if hi_c - lo_c > 0.025 * hi_c:
                cut = (lo_c + hi_c) / 2
                for c in todo:                              # the slow cluster's upper tail gets more chances
                    tries = 0
                    while lo_c + 0.5 * (cut - lo_c) < rate[c] <= cut and tries < 3:
                        rate[c] = max(rate[c], measure(ctx, c, 8))
                        tries += 1
            else:
                cut = float("-inf")                         # one cluster: everything shares the reference's rank
            _B.gxpo_destroy(ctx)
            same = [c for c in todo if rate[c] > cut or c == ref]
            for c in same:
                labels[c] = next_label
            if verbose:
                print(f"[hbm_arena] reference chunk {ref}: {len(same)} of {len(todo)} chunks share its rank "
                      f"(cluster centres {lo_c:.0f} / {hi_c:.0f} GB/s)", file=sys.stderr, flush=True)
            # next reference: the slowest chunk still unlabelled, the one least likely to be a straggler of this rank
            # (a straggler as reference would make everything else look like one foreign cluster)
            todo = sorted((c for c in todo if labels[c] < 0), key=lambda c: rate[c])
            next_label += 1
        for c in todo:                                      # more clusters than ranks can be: lump the rest together
            labels[c] = next_label
        grads.clear()
        torch.cuda.synchronize(self.device)
        self._unmap_all()
        self.labels = labels
        return labels

    # ---- buffers ---------------------------------------------------------------------------------------
    def build(self, specs: Sequence[dict], scatter: bool = True, tune: int = 0, verbose: bool = False) -> Dict[str, torch.Tensor]:
        """specs: dicts with name, numel, dtype, phase_bytes, group ('update', 'read' or 'write').  All buffers
        index the same elements.  Slab by slab, the chunks of every 'update' and 'read' buffer come from one rank;
        'write' buffers take theirs from another rank where there is room.  With `tune` > 0 the chunks of theta, m, v
        are then chosen by measurement, the best of `tune` candidate triples per chunk position.  Returns name -> tensor."""
        if not self.labels:
            raise ArenaUnavailable("classify() has not run")
        cb = self.chunk_bytes
        available = [i for i, h in enumerate(self.handles) if h is not None]
        plan, self.slab_rank = plan_chunks(self.labels, [dict(s, itemsize=torch.empty((), dtype=s["dtype"]).element_size()) for s in specs],
                                           cb, available, scatter)
        self.tuned = None
        if tune > 0:
            self._tune_updates(plan, specs, available, tune, verbose)
        out = {}
        for s in specs:
            chunks = plan[s["name"]]
            va = self._reserve(len(chunks) * cb)
            for k, c in enumerate(chunks):
                self._map(va + k * cb, c)
            out[s["name"]] = self._tensor(va + s.get("phase_bytes", 0), s["numel"], s["dtype"])
        used = {c for chunks in plan.values() for c in chunks}
        assert sum(len(chunks) for chunks in plan.values()) == len(used)
        hip = _runtime()
        for i, h in enumerate(self.handles):               # give back what the buffers did not need
            if i not in used and h is not None:
                hip.hipMemRelease(h)
                self.handles[i] = None
        self.plan = plan
        return out

    def _tune_updates(self, plan, specs, available, candidates: int, verbose: bool):
        """Which three chunks hold theta, m and v of one chunk position decides the pass rate more than anything
        else inside a rank: triples drawn at random from one rank measured between 75 % and 83.5 % of peak on the
        fallback step (standard deviation one point), and no rule in the chunk numbers predicts it.  So they are
        chosen by measurement: per position, `candidates` random triples from the rank's pool (the chunks planned
        for theta, m, v there plus the spare ones) are timed with the engine's fallback step on windows at the
        start of the chunks, against the chunks planned there for the first and the last gradient stream (what the
        fused pass and the fallback step read, and what the slow step reads), and the best triple is kept.
        With the second buffer set of the alternating schedule (theta_probe, m_alt, v_alt as 'update' buffers of
        set 1) each set's triple is chosen while it is the written one: set 1 against set 0's planned triple and
        the first gradient of set 0, then set 0 against the chosen set 1 and the first gradient of set 1.
        Edits `plan` in place; leaves it alone when the buffers are not the AdamW set."""
        cb, labels = self.chunk_bytes, self.labels
        upd = [[s for s in specs if s["group"] == "update" and s.get("set", 0) == k] for k in (0, 1)]
        reads = [[s for s in specs if s["group"] == "read" and s.get("set", 0) == k] for k in (0, 1)]
        alternating = [s["name"] for s in upd[1]] == ["theta_probe", "m_alt", "v_alt"]
        every = upd[0] + upd[1] + reads[0] + reads[1]
        if [s["name"] for s in upd[0]] != ["theta", "m", "v"] or (upd[1] and not alternating) or not reads[0] \
                or (alternating and not reads[1]) or any(s["dtype"] != torch.float32 for s in upd[0] + upd[1]) \
                or any(s.get("phase_bytes", 0) >= 65536 for s in every) or len({s["dtype"] for s in reads[0] + reads[1]}) != 1:
            return
        g_size = torch.empty((), dtype=reads[0][0]["dtype"]).element_size()
        E = (cb - 65536) // 4
        n_pos = min(len(plan[s["name"]]) for s in upd[0] + upd[1])
        va = self._reserve(len(self.handles) * cb)
        for c in available:
            self._map(va + c * cb, c)
        cfg = _B.make_config(K=2, lr=1e-9, weight_decay=0.0, delta=0.0, grad_dtype="f32" if g_size == 4 else "bf16")
        f32 = lambda c, s: self._tensor(va + c * cb + s.get("phase_bytes", 0), E, torch.float32)

        def gradient_window(g_spec, k):
            at = k * (cb // 4) * g_size                                          # where position k starts in the gradient buffer
            chunk = plan[g_spec["name"]][min(at // cb, len(plan[g_spec["name"]]) - 1)]
            g = self._tensor(va + chunk * cb + min(at % cb, cb - E * g_size), E, g_spec["dtype"])
            g.normal_(std=0.05)
            return g

        def timed(ctx, g, before_each=None):
            if before_each:
                before_each()
            _B.gxpo_fallback_step(ctx, [g])
            best = float("inf")
            for _ in range(2):                                                   # disturbances only slow a measurement down
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for _ in range(3):
                    if before_each:
                        before_each()
                    _B.gxpo_fallback_step(ctx, [g])
                b.record()
                b.synchronize()
                best = min(best, a.elapsed_time(b) / 3)
            return best

        def pools_and_positions(which):
            """Per chunk position the class the triple of set `which` is planned in (None where its three chunks
            disagree), and per class the chunks a triple may be drawn from: the planned ones plus the spare ones."""
            names = [s["name"] for s in upd[which]]
            used = {c for chunks in plan.values() for c in chunks}
            pools: Dict[int, List[int]] = {}
            for c in available:
                if c not in used:
                    pools.setdefault(labels[c], []).append(c)
            positions = []
            for k in range(n_pos):
                labs = {labels[plan[n][k]] for n in names}
                lab = labs.pop() if len(labs) == 1 else None
                positions.append(lab)
                if lab is not None:
                    pools.setdefault(lab, []).extend(plan[n][k] for n in names)
            for lab in pools:
                pools[lab].sort()
            return names, pools, positions

        stats = []
        cache = {}
        try:
            if not alternating:
                names, pools, positions = pools_and_positions(0)
                g_specs = [reads[0][0]] + ([reads[0][-1]] if len(reads[0]) > 1 else [])

                def measure(k, tup):
                    if cache.get("k") != k:
                        cache.update(k=k, gs=[gradient_window(g, k) for g in g_specs])
                    th, m, v = (f32(c, s) for c, s in zip(tup, upd[0]))
                    th.normal_(std=0.02), m.zero_(), v.fill_(1e-4)
                    ctx = _B.gxpo_init(cfg, [dict(theta=th, m=m, v=v)])
                    st = _B.gxpo_get_state(ctx)
                    st.s_star = 0
                    _B.gxpo_set_state(ctx, st)
                    total_ms = sum(timed(ctx, g) for g in cache["gs"])
                    _B.gxpo_destroy(ctx)
                    return len(g_specs) * (24.0 + g_size) * E / total_ms / 1e6

                tuples, seen = choose_tuples(pools, positions, 3, candidates, measure)
                stats.append(("theta, m, v", seen))
                for k, tup in enumerate(tuples):
                    if tup is not None:
                        for n, c in zip(names, tup):
                            plan[n][k] = c
            else:
                for written in (1, 0):                                           # set 1 first: it is written by the first pass of a step
                    names, pools, positions = pools_and_positions(written)
                    g_spec = reads[1 - written][0]                               # a gradient next to the set that is read

                    def measure(k, tup, written=written, g_spec=g_spec):
                        if cache.get("k") != (written, k):
                            cache.update(k=(written, k), g=gradient_window(g_spec, k))
                        chunks = {written: tup, 1 - written: [plan[s["name"]][k] for s in upd[1 - written]]}
                        (th, m, v), (th1, m1, v1) = ([f32(c, s) for c, s in zip(chunks[w], upd[w])] for w in (0, 1))
                        src = (th, m, v) if written == 1 else (th1, m1, v1)
                        src[0].normal_(std=0.02), src[1].zero_(), src[2].fill_(1e-4)
                        ctx = _B.gxpo_init(cfg, [dict(theta=th, m=m, v=v, theta_probe=th1, m_alt=m1, v_alt=v1)])
                        st = _B.gxpo_get_state(ctx)
                        st.s_star, st.current_set = 0, 1 - written

                        def rewind():                                            # every timed step reads the same set again
                            _B.gxpo_set_state(ctx, st)

                        ms = timed(ctx, cache["g"], rewind)
                        _B.gxpo_destroy(ctx)
                        return (24.0 + g_size) * E / ms / 1e6

                    tuples, seen = choose_tuples(pools, positions, 3, candidates, measure, seed=written)
                    stats.append((", ".join(names), seen))
                    for k, tup in enumerate(tuples):
                        if tup is not None:
                            for n, c in zip(names, tup):
                                plan[n][k] = c
        finally:
            cache.clear()
            torch.cuda.synchronize(self.device)
            self._unmap_all()
        rated = [(what, [r for r in seen if r]) for what, seen in stats]
        rated = [(what, r) for what, r in rated if r]
        if rated:
            allr = [r for _, rs in rated for r in rs]
            self.tuned = {"positions": len(rated[0][1]), "candidates": candidates,
                          "mean_gbps": round(sum(sum(r) for r in allr) / sum(len(r) for r in allr)),
                          "chosen_gbps": round(sum(max(r) for r in allr) / len(allr))}
            if verbose:
                for what, rs in rated:
                    print(f"[hbm_arena] {what} chosen by measurement at {len(rs)} chunk positions: candidates average "
                          f"{round(sum(sum(r) for r in rs) / sum(len(r) for r in rs))} GB/s on the fallback step, chosen ones "
                          f"{round(sum(max(r) for r in rs) / len(rs))} GB/s", file=sys.stderr, flush=True)

    def close(self):
        if self._closed:
            return
        self._closed = True
        try:
            torch.cuda.synchronize(self.device)
        except Exception:
            pass
        self._unmap_all()
        hip = _runtime()
        for i, h in enumerate(self.handles):
            if h is not None:
                hip.hipMemRelease(h)
                self.handles[i] = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
