"""ctypes binding of libgxpo.so: argument marshalling only.

Every function here has the name and the meaning of the C entry point it wraps
(include/gxpo.h); nothing of the update rule is computed in Python.  PyTorch
appears only as the owner of device memory and streams: tensors are turned
into raw device pointers, the current torch stream is passed as the HIP stream.

Importing this module fails loudly if the library has not been built
(`python -m paper_2605_06755_amd.build`); there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import math
import os
from typing import List, Optional, Sequence

import torch  # noqa: F401  (loads the process-wide HIP runtime before libgxpo.so binds to it)

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libgxpo.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build the HIP library first with "
        "`python -m paper_2605_06755_amd.build` (there is no CPU fallback)")
_lib = ctypes.CDLL(LIB_PATH)

# ---- enums ---------------------------------------------------------------------------------
GXPO_OK = 0
GXPO_ERR_INVALID_ARG = -1
GXPO_ERR_BAD_STATE = -2
GXPO_ERR_ALIGNMENT = -3
GXPO_ERR_UNSUPPORTED = -4
GXPO_ERR_HIP = -5
GXPO_ERR_NOMEM = -6
GXPO_OPT_GD, GXPO_OPT_ADAMW = 0, 1
GXPO_GRAD_F32, GXPO_GRAD_BF16 = 0, 1
GXPO_COPY_AT_PROBE, GXPO_COPY_AT_TILDE, GXPO_COPY_AT_FINAL = 1, 2, 4
GXPO_PHASE_IDLE, GXPO_PHASE_FAST1, GXPO_PHASE_FAST2, GXPO_PHASE_REPOSITIONED, GXPO_PHASE_SLOW_DONE = range(5)
GXPO_MAX_WINDOW = 256
GXPO_BUF_THETA, GXPO_BUF_THETA_PROBE, GXPO_BUF_M, GXPO_BUF_V, GXPO_BUF_MODEL_COPY, GXPO_BUF_GRAD = range(6)

EXPORTED_SYMBOLS = [
    "gxpo_init", "gxpo_destroy", "gxpo_fast_steps", "gxpo_extrapolate", "gxpo_slow_step", "gxpo_gate",
    "gxpo_fallback_step", "gxpo_tensor_norms", "gxpo_get_diagnostics", "gxpo_get_state", "gxpo_set_state", "gxpo_last_error",
    "gxpo_validate_config", "gxpo_host_gate_step", "gxpo_plan_blocks", "gxpo_stream_copy", "gxpo_update_config",
    "gxpo_set_tensor_options", "gxpo_layout_hint", "gxpo_slow_step_noalloc", "gxpo_current_params",
]


# ---- structs (mirror include/gxpo.h) ----------------------------------------------------------
class gxpo_tensor(ctypes.Structure):
    _fields_ = [("numel", ctypes.c_uint64), ("theta", ctypes.c_void_p), ("theta_probe", ctypes.c_void_p),
                ("m", ctypes.c_void_p), ("v", ctypes.c_void_p), ("model_copy", ctypes.c_void_p),
                ("m_alt", ctypes.c_void_p), ("v_alt", ctypes.c_void_p)]


class gxpo_config(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("optimizer", ctypes.c_uint32), ("grad_dtype", ctypes.c_uint32),
                ("K", ctypes.c_uint32), ("fuse_step2", ctypes.c_uint32), ("copy_mask", ctypes.c_uint32),
                ("window", ctypes.c_uint32), ("gate_min_count", ctypes.c_uint32), ("gate_ddof", ctypes.c_uint32),
                ("diagnostics", ctypes.c_uint32), ("explicit_steps", ctypes.c_uint32),
                ("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("adam_eps", ctypes.c_double), ("weight_decay", ctypes.c_double),
                ("alpha", ctypes.c_double), ("delta", ctypes.c_double), ("r_max", ctypes.c_double),
                ("clip_norm", ctypes.c_double), ("tau", ctypes.c_double), ("gate_eps", ctypes.c_double)]


class gxpo_tensor_options(ctypes.Structure):
    _fields_ = [("lr_scale", ctypes.c_double), ("weight_decay_scale", ctypes.c_double)]


class gxpo_gate_info(ctypes.Structure):
    _fields_ = [("norm", ctypes.c_double), ("mu", ctypes.c_double), ("sigma", ctypes.c_double), ("z", ctypes.c_double),
                ("evaluated", ctypes.c_int32), ("tripped", ctypes.c_int32), ("s_star", ctypes.c_int64),
                ("t", ctypes.c_int64)]


class gxpo_diagnostics(ctypes.Structure):
    _fields_ = [("norm_g0", ctypes.c_double), ("norm_g1", ctypes.c_double), ("norm_g_slow", ctypes.c_double),
                ("cos_g0_g_slow", ctypes.c_double), ("retention_mean", ctypes.c_double), ("retention_std", ctypes.c_double),
                ("scale_mean", ctypes.c_double), ("inactive_fraction", ctypes.c_double),
                ("displacement_ratio", ctypes.c_double), ("t", ctypes.c_int64)]


class gxpo_state(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("phase", ctypes.c_uint32), ("t", ctypes.c_int64),
                ("optim_steps", ctypes.c_int64), ("s_star", ctypes.c_int64), ("backward_passes", ctypes.c_int64),
                ("window_len", ctypes.c_uint32), ("current_set", ctypes.c_uint32),
                ("window", ctypes.c_double * GXPO_MAX_WINDOW)]


_ctx_p = ctypes.c_void_p
_ptr_list = ctypes.POINTER(ctypes.c_void_p)

_lib.gxpo_init.restype = ctypes.c_int
_lib.gxpo_init.argtypes = [ctypes.POINTER(_ctx_p), ctypes.POINTER(gxpo_config), ctypes.POINTER(gxpo_tensor), ctypes.c_uint32]
_lib.gxpo_destroy.restype = None
_lib.gxpo_destroy.argtypes = [_ctx_p]
_lib.gxpo_fast_steps.restype = ctypes.c_int
_lib.gxpo_fast_steps.argtypes = [_ctx_p, ctypes.c_int, _ptr_list, ctypes.c_void_p]
_lib.gxpo_extrapolate.restype = ctypes.c_int
_lib.gxpo_extrapolate.argtypes = [_ctx_p, _ptr_list, _ptr_list, ctypes.c_void_p]
_lib.gxpo_slow_step.restype = ctypes.c_int
_lib.gxpo_slow_step.argtypes = [_ctx_p, _ptr_list, ctypes.c_void_p]
_lib.gxpo_gate.restype = ctypes.c_int
_lib.gxpo_gate.argtypes = [_ctx_p, ctypes.POINTER(gxpo_gate_info), ctypes.c_void_p]
_lib.gxpo_fallback_step.restype = ctypes.c_int
_lib.gxpo_fallback_step.argtypes = [_ctx_p, _ptr_list, ctypes.c_void_p]
_lib.gxpo_tensor_norms.restype = ctypes.c_int
_lib.gxpo_tensor_norms.argtypes = [_ctx_p, ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
_lib.gxpo_get_diagnostics.restype = ctypes.c_int
_lib.gxpo_get_diagnostics.argtypes = [_ctx_p, ctypes.POINTER(gxpo_diagnostics), ctypes.c_void_p]
_lib.gxpo_current_params.argtypes = [_ctx_p, ctypes.POINTER(ctypes.c_void_p)]
_lib.gxpo_current_params.restype = ctypes.c_int
_lib.gxpo_get_state.restype = ctypes.c_int
_lib.gxpo_get_state.argtypes = [_ctx_p, ctypes.POINTER(gxpo_state)]
_lib.gxpo_set_state.restype = ctypes.c_int
_lib.gxpo_set_state.argtypes = [_ctx_p, ctypes.POINTER(gxpo_state)]
_lib.gxpo_update_config.restype = ctypes.c_int
_lib.gxpo_update_config.argtypes = [_ctx_p, ctypes.POINTER(gxpo_config)]
_lib.gxpo_set_tensor_options.restype = ctypes.c_int
_lib.gxpo_set_tensor_options.argtypes = [_ctx_p, ctypes.POINTER(gxpo_tensor_options)]
_lib.gxpo_last_error.restype = ctypes.c_char_p
_lib.gxpo_last_error.argtypes = [_ctx_p]
_lib.gxpo_validate_config.restype = ctypes.c_int
_lib.gxpo_validate_config.argtypes = [ctypes.POINTER(gxpo_config), ctypes.c_char_p, ctypes.c_size_t]
_lib.gxpo_host_gate_step.restype = ctypes.c_int
_lib.gxpo_host_gate_step.argtypes = [ctypes.POINTER(gxpo_config), ctypes.POINTER(gxpo_state), ctypes.c_double,
                                     ctypes.POINTER(gxpo_gate_info)]
_lib.gxpo_plan_blocks.restype = ctypes.c_int
_lib.gxpo_plan_blocks.argtypes = [ctypes.POINTER(ctypes.c_uint64), ctypes.c_uint32,
                                  ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(ctypes.c_uint32)]
_lib.gxpo_layout_hint.restype = ctypes.c_int
_lib.gxpo_layout_hint.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint64)]
_lib.gxpo_slow_step_noalloc.restype = ctypes.c_int
_lib.gxpo_slow_step_noalloc.argtypes = [ctypes.POINTER(gxpo_config), ctypes.POINTER(gxpo_tensor), ctypes.c_int64, ctypes.c_void_p,
                                        ctypes.c_void_p, ctypes.c_void_p]
GXPO_NOALLOC_MAX_NUMEL = 1 << 28
_lib.gxpo_stream_copy.restype = ctypes.c_int
_lib.gxpo_stream_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p]


class GxpoError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"gxpo error {code}: {message}")
        self.code = code
        self.message = message


def make_config(*, optimizer="adamw", grad_dtype="f32", K=8, fuse_step2=True, copy_mask=7, window=10,
                gate_min_count=0, gate_ddof=0, diagnostics=False, explicit_steps=0, lr=1e-6, beta1=0.9, beta2=0.999,
                adam_eps=1e-8, weight_decay=0.01, alpha=0.5, delta=1e-8, r_max=math.inf, clip_norm=0.0, tau=3.0,
                gate_eps=1e-8) -> gxpo_config:
    c = gxpo_config()
    c.struct_size = ctypes.sizeof(gxpo_config)
    c.optimizer = {"gd": GXPO_OPT_GD, "adamw": GXPO_OPT_ADAMW}.get(optimizer, optimizer)
    c.grad_dtype = {"f32": GXPO_GRAD_F32, "bf16": GXPO_GRAD_BF16}.get(grad_dtype, grad_dtype)
    c.K, c.fuse_step2, c.copy_mask = int(K), int(bool(fuse_step2)), int(copy_mask)
    c.window, c.gate_min_count, c.gate_ddof = int(window), int(gate_min_count), int(gate_ddof)
    c.diagnostics, c.explicit_steps = int(diagnostics), int(explicit_steps)
    c.lr, c.beta1, c.beta2, c.adam_eps, c.weight_decay = lr, beta1, beta2, adam_eps, weight_decay
    c.alpha, c.delta, c.r_max, c.clip_norm, c.tau, c.gate_eps = alpha, delta, r_max, clip_norm, tau, gate_eps
    return c


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return int(stream) or None


def _dev_ptr(t: Optional[torch.Tensor], dtype, numel) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous() or t.numel() != numel:
        raise ValueError(f"expected a contiguous device tensor of dtype {dtype} with {numel} elements, got "
                         f"{t.dtype} {tuple(t.shape)} on {t.device}")
    return t.data_ptr()


class Context:
    """Owner of a gxpo_ctx*.  Keeps the tensors it was built from alive."""

    def __init__(self, handle: int, cfg: gxpo_config, keep):
        self.handle = _ctx_p(handle)
        self.cfg = cfg
        self.n_tensors = len(keep)
        self._keep = keep
        self._numels = [k["theta"].numel() for k in keep]
        self._grad_dtype = torch.float32 if cfg.grad_dtype == GXPO_GRAD_F32 else torch.bfloat16
        self._last_grads = {}

    def close(self):
        if self.handle:
            _lib.gxpo_destroy(self.handle)
            self.handle = _ctx_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _grad_list(self, grads, role: str):
        if isinstance(grads, GradList):
            if grads.ctx is not self:
                raise ValueError("this GradList was prepared for another context")
            self._last_grads[role] = grads
            return grads.array
        if len(grads) != self.n_tensors:
            raise ValueError(f"expected {self.n_tensors} gradient tensors, got {len(grads)}")
        arr = (ctypes.c_void_p * self.n_tensors)(*[_dev_ptr(g, self._grad_dtype, n) for g, n in zip(grads, self._numels)])
        self._last_grads[role] = list(grads)        # keep alive while kernels may read them
        return arr

    def _check(self, rc: int):
        if rc != GXPO_OK:
            raise GxpoError(rc, _lib.gxpo_last_error(self.handle).decode())


class GradList:
    """A gradient list marshalled once (pointer array built and checked), for callers that
    hand the same buffers in every step: with hundreds of small tensors, rebuilding the
    pointer array in Python on every call costs more than the kernels."""

    def __init__(self, ctx: Context, grads: Sequence[torch.Tensor]):
        self.ctx = ctx
        self.tensors = list(grads)
        self.array = ctx._grad_list(self.tensors, "prepared")


def gxpo_init(cfg: gxpo_config, tensors: Sequence[dict]) -> Context:
    """tensors: one dict per parameter tensor with torch tensors under the keys
    theta, theta_probe, and optionally m, v, model_copy, m_alt, v_alt."""
    n = len(tensors)
    arr = (gxpo_tensor * max(n, 1))()
    for i, t in enumerate(tensors):
        numel = t["theta"].numel()
        arr[i].numel = numel
        arr[i].theta = _dev_ptr(t["theta"], torch.float32, numel)
        arr[i].theta_probe = _dev_ptr(t.get("theta_probe"), torch.float32, numel)
        arr[i].m = _dev_ptr(t.get("m"), torch.float32, numel)
        arr[i].v = _dev_ptr(t.get("v"), torch.float32, numel)
        arr[i].model_copy = _dev_ptr(t.get("model_copy"), torch.bfloat16, numel)
        arr[i].m_alt = _dev_ptr(t.get("m_alt"), torch.float32, numel)
        arr[i].v_alt = _dev_ptr(t.get("v_alt"), torch.float32, numel)
    handle = _ctx_p(None)
    rc = _lib.gxpo_init(ctypes.byref(handle), ctypes.byref(cfg), arr, n)
    if rc != GXPO_OK:
        raise GxpoError(rc, _lib.gxpo_last_error(None).decode())
    return Context(handle.value, cfg, [dict(t) for t in tensors])


def gxpo_destroy(ctx: Context) -> None:
    ctx.close()


def gxpo_fast_steps(ctx: Context, which: int, grads: Sequence[torch.Tensor], stream=None) -> None:
    ctx._check(_lib.gxpo_fast_steps(ctx.handle, which, ctx._grad_list(grads, f"fast{which}"), _stream_ptr(stream)))


def gxpo_extrapolate(ctx: Context, g0=None, g1=None, stream=None) -> None:
    """g0, g1 may be None only for a context with explicit_steps (reposition without extrapolation)."""
    a0 = ctx._grad_list(g0, "ex0") if g0 is not None else None
    a1 = ctx._grad_list(g1, "ex1") if g1 is not None else None
    ctx._check(_lib.gxpo_extrapolate(ctx.handle, a0, a1, _stream_ptr(stream)))


def gxpo_slow_step(ctx: Context, g_slow: Sequence[torch.Tensor], stream=None) -> None:
    ctx._check(_lib.gxpo_slow_step(ctx.handle, ctx._grad_list(g_slow, "slow"), _stream_ptr(stream)))


def gxpo_gate(ctx: Context, stream=None) -> gxpo_gate_info:
    info = gxpo_gate_info()
    ctx._check(_lib.gxpo_gate(ctx.handle, ctypes.byref(info), _stream_ptr(stream)))
    return info


def gxpo_fallback_step(ctx: Context, g0: Sequence[torch.Tensor], stream=None) -> None:
    ctx._check(_lib.gxpo_fallback_step(ctx.handle, ctx._grad_list(g0, "fallback"), _stream_ptr(stream)))


def gxpo_tensor_norms(ctx: Context, stream=None) -> List[float]:
    out = (ctypes.c_double * ctx.n_tensors)()
    ctx._check(_lib.gxpo_tensor_norms(ctx.handle, out, _stream_ptr(stream)))
    return list(out)


def gxpo_get_diagnostics(ctx: Context, stream=None) -> gxpo_diagnostics:
    d = gxpo_diagnostics()
    ctx._check(_lib.gxpo_get_diagnostics(ctx.handle, ctypes.byref(d), _stream_ptr(stream)))
    return d


def gxpo_current_params(ctx: Context) -> List[torch.Tensor]:
    """The tensors (out of the ones the context was built from) that hold the current iterate."""
    out = (ctypes.c_void_p * ctx.n_tensors)()
    ctx._check(_lib.gxpo_current_params(ctx.handle, out))
    found = []
    for t, ptr in zip(ctx._keep, out):
        found.append(next(t[k] for k in ("theta", "theta_probe") if t.get(k) is not None and t[k].data_ptr() == ptr))
    return found


def gxpo_get_state(ctx: Context) -> gxpo_state:
    st = gxpo_state()
    ctx._check(_lib.gxpo_get_state(ctx.handle, ctypes.byref(st)))
    return st


def gxpo_set_state(ctx: Context, st: gxpo_state) -> None:
    ctx._check(_lib.gxpo_set_state(ctx.handle, ctypes.byref(st)))


def gxpo_update_config(ctx: Context, cfg: gxpo_config) -> None:
    ctx._check(_lib.gxpo_update_config(ctx.handle, ctypes.byref(cfg)))
    ctx.cfg = cfg


def gxpo_set_tensor_options(ctx: Context, lr_scale: Sequence[float], weight_decay_scale: Sequence[float]) -> None:
    if len(lr_scale) != ctx.n_tensors or len(weight_decay_scale) != ctx.n_tensors:
        raise ValueError(f"expected {ctx.n_tensors} multipliers of each kind")
    arr = (gxpo_tensor_options * ctx.n_tensors)()
    for i, (a, b) in enumerate(zip(lr_scale, weight_decay_scale)):
        arr[i].lr_scale, arr[i].weight_decay_scale = float(a), float(b)
    ctx._check(_lib.gxpo_set_tensor_options(ctx.handle, arr))


def gxpo_last_error(ctx: Optional[Context] = None) -> str:
    return _lib.gxpo_last_error(ctx.handle if ctx else None).decode()


def gxpo_validate_config(cfg: gxpo_config):
    """Returns (status, message)."""
    buf = ctypes.create_string_buffer(256)
    rc = _lib.gxpo_validate_config(ctypes.byref(cfg), buf, 256)
    return rc, buf.value.decode()


def gxpo_host_gate_step(cfg: gxpo_config, state: gxpo_state, norm: float) -> gxpo_gate_info:
    info = gxpo_gate_info()
    rc = _lib.gxpo_host_gate_step(ctypes.byref(cfg), ctypes.byref(state), float(norm), ctypes.byref(info))
    if rc != GXPO_OK:
        raise GxpoError(rc, "gxpo_host_gate_step rejected its arguments")
    return info


def new_state() -> gxpo_state:
    st = gxpo_state()
    st.struct_size = ctypes.sizeof(gxpo_state)
    st.s_star = -1
    return st


def gxpo_plan_blocks(numels: Sequence[int]):
    """Returns (block_start list of len n + 1, elems_per_block)."""
    n = len(numels)
    arr = (ctypes.c_uint64 * max(n, 1))(*numels)
    out = (ctypes.c_uint32 * (n + 1))()
    epb = ctypes.c_uint32(0)
    rc = _lib.gxpo_plan_blocks(arr, n, out, ctypes.byref(epb))
    if rc != GXPO_OK:
        raise GxpoError(rc, "gxpo_plan_blocks rejected its arguments")
    return list(out), epb.value


def gxpo_layout_hint(buffer_kind: int):
    """Returns (phase_bytes, period_bytes) for a GXPO_BUF_* kind."""
    phase, period = ctypes.c_uint64(0), ctypes.c_uint64(0)
    rc = _lib.gxpo_layout_hint(int(buffer_kind), ctypes.byref(phase), ctypes.byref(period))
    if rc != GXPO_OK:
        raise GxpoError(rc, "gxpo_layout_hint rejected its arguments")
    return phase.value, period.value


def gxpo_slow_step_noalloc(cfg: gxpo_config, tensor: dict, optim_step: int, g_slow: torch.Tensor, sum_sq_out: torch.Tensor,
                           stream=None) -> None:
    """tensor: dict with theta and optionally m, v, model_copy (torch tensors); sum_sq_out: one float64 on the device."""
    numel = tensor["theta"].numel()
    rec = gxpo_tensor()
    rec.numel = numel
    rec.theta = _dev_ptr(tensor["theta"], torch.float32, numel)
    rec.m = _dev_ptr(tensor.get("m"), torch.float32, numel)
    rec.v = _dev_ptr(tensor.get("v"), torch.float32, numel)
    rec.model_copy = _dev_ptr(tensor.get("model_copy"), torch.bfloat16, numel)
    gdt = torch.float32 if cfg.grad_dtype == GXPO_GRAD_F32 else torch.bfloat16
    rc = _lib.gxpo_slow_step_noalloc(ctypes.byref(cfg), ctypes.byref(rec), int(optim_step), _dev_ptr(g_slow, gdt, numel),
                                     _dev_ptr(sum_sq_out, torch.float64, 1), _stream_ptr(stream))
    if rc != GXPO_OK:
        raise GxpoError(rc, _lib.gxpo_last_error(None).decode())


def gxpo_stream_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("size mismatch")
    rc = _lib.gxpo_stream_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream_ptr(stream))
    if rc != GXPO_OK:
        raise GxpoError(rc, _lib.gxpo_last_error(None).decode())
