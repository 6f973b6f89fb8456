"""Seeded synthetic workloads: parameter layouts and a noisy-quadratic "trainer".

This module stands in for everything the update engine does not own: the
policy's parameter shapes and the loss whose gradients the trainer hands over
three times per active step.  It holds none of the update rule's arithmetic
(no optimizer step, no ratio, no extrapolation, no gate); both the HIP engine's
tests / bench and the CPU oracle's tests draw their inputs from here.

The loss is the diagonal quadratic of the paper's surrogate analysis
(Section 2.4 corollary; Appendix A.6), shifted to a minimiser theta_star and
optionally perturbed by additive gradient noise:

    L(theta) = 1/2 sum_i h_i (theta_i - theta_star_i)^2
    g(theta) = h * (theta - theta_star) + sigma * xi

Within one training step the three gradients are taken on the same batch
(Section 2, first paragraph: rollouts, rewards and advantages are reused), so
one noise draw xi_t is shared by g0, g1 and g_slow of step t and a fresh one
is drawn for the next step.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Tuple

import torch

# ---------------------------------------------------------------------------
# parameter layouts
# ---------------------------------------------------------------------------
QWEN25_1P5B_PARAMS = 1_540_000_000      # flat stand-in for Qwen2.5-1.5B
QWEN25_7B_PARAMS = 7_600_000_000        # flat stand-in for Qwen2.5-7B
GATE_STRESS_PARAMS = 3_200_000_000


def llama31_8b_layout() -> List[Tuple[str, int]]:
    """(name, numel) of the ragged Llama-3.1-8B tensor list: 290 tensors.

    Embedding and output head 128256 x 4096; 32 decoder layers, each with
    q/o 4096 x 4096, k/v 1024 x 4096, gate/up 14336 x 4096, down 4096 x 14336
    and two 4096-element RMSNorm vectors.
    """
    out = [("embed_tokens", 128256 * 4096)]
    for layer in range(32):
        p = f"layers.{layer}."
        out += [
            (p + "input_layernorm", 4096),
            (p + "q_proj", 4096 * 4096),
            (p + "k_proj", 1024 * 4096),
            (p + "v_proj", 1024 * 4096),
            (p + "o_proj", 4096 * 4096),
            (p + "post_attention_layernorm", 4096),
            (p + "gate_proj", 14336 * 4096),
            (p + "up_proj", 14336 * 4096),
            (p + "down_proj", 4096 * 14336),
        ]
    out.append(("lm_head", 128256 * 4096))
    return out


def qwen25_7b_lora_layout(rank: int = 128) -> List[Tuple[str, int]]:
    """(name, numel) of rank-`rank` LoRA adapters on the q, k, v, o projections of a
    Qwen2.5-7B-shaped model (hidden 3584, 28 layers, 28 query heads and 4 key/value heads
    of dimension 128): 224 small tensors, 80,740,352 parameters at rank 128."""
    hidden, kv = 3584, 4 * 128
    out = []
    for layer in range(28):
        for proj, d_out in (("q", hidden), ("k", kv), ("v", kv), ("o", hidden)):
            out.append((f"layers.{layer}.{proj}_proj.lora_A", rank * hidden))
            out.append((f"layers.{layer}.{proj}_proj.lora_B", d_out * rank))
    return out


def scaled_layout(layout: List[Tuple[str, int]], divisor: int, multiple: int = 1) -> List[Tuple[str, int]]:
    """Same tensor list with every numel divided (floor, at least 1, then
    rounded down to `multiple` when that leaves something): keeps the ragged
    mix of huge and tiny tensors at a size a CPU can check."""
    out = []
    for name, n in layout:
        k = max(1, n // divisor)
        if multiple > 1 and k >= multiple:
            k -= k % multiple
        out.append((name, k))
    return out


# ---------------------------------------------------------------------------
# noisy diagonal quadratic
# ---------------------------------------------------------------------------
@dataclass
class QuadraticProblem:
    h: torch.Tensor            # curvatures, fp32
    theta_star: torch.Tensor   # minimiser, fp32
    theta_0: torch.Tensor      # starting point, fp32
    sigma: float               # gradient-noise scale
    seed: int

    @property
    def numel(self) -> int:
        return self.h.numel()


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def make_quadratic(numel: int, seed: int, *, h_dist: str, h_lo: float, h_hi: float,
                   theta_std: float, sigma: float, device="cpu") -> QuadraticProblem:
    """h ~ U[h_lo, h_hi] ('uniform') or LogUniform[h_lo, h_hi] ('loguniform');
    theta_star, theta_0 ~ N(0, theta_std^2).  All fp32, all from `seed`."""
    gen = _gen(device, seed)
    u = torch.rand(numel, generator=gen, device=device, dtype=torch.float32)
    if h_dist == "uniform":
        h = u.mul_(h_hi - h_lo).add_(h_lo)
    elif h_dist == "loguniform":
        h = u.mul_(math.log(h_hi) - math.log(h_lo)).add_(math.log(h_lo)).exp_()
    else:
        raise ValueError(h_dist)
    theta_star = torch.randn(numel, generator=gen, device=device, dtype=torch.float32).mul_(theta_std)
    theta_0 = torch.randn(numel, generator=gen, device=device, dtype=torch.float32).mul_(theta_std)
    return QuadraticProblem(h, theta_star, theta_0, sigma, seed)


def surrogate_problem(numel: int = 1 << 20, seed: int = 0, device="cpu") -> QuadraticProblem:
    """Plain-GD quadratic surrogate: h ~ U[0.1, 1], theta ~ N(0, 1), no noise."""
    return make_quadratic(numel, seed, h_dist="uniform", h_lo=0.1, h_hi=1.0,
                          theta_std=1.0, sigma=0.0, device=device)


def policy_problem(numel: int, seed: int, sigma: float = 0.05, device="cpu") -> QuadraticProblem:
    """LLM-policy-like stand-in: h ~ LogUniform[1e-3, 1], theta ~ N(0, 0.02^2),
    gradient noise sigma * N(0, 1)."""
    return make_quadratic(numel, seed, h_dist="loguniform", h_lo=1e-3, h_hi=1.0,
                          theta_std=0.02, sigma=sigma, device=device)


def step_noise(problem: QuadraticProblem, step: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """The noise draw xi_t of training step `step` (shared by that step's
    three gradients).  Deterministic in (problem.seed, step)."""
    dev = problem.h.device
    gen = _gen(dev, (problem.seed + 1) * 1_000_003 + step)
    if out is None:
        return torch.randn(problem.numel, generator=gen, device=dev, dtype=torch.float32)
    return out.normal_(generator=gen)


def quadratic_grad(problem: QuadraticProblem, theta: torch.Tensor, noise: torch.Tensor | None,
                   sigma: float | None = None, out_dtype=torch.float32) -> torch.Tensor:
    """g = h * (theta - theta_star) + sigma * noise, computed in theta's dtype
    (fp32 on the GPU side, fp64 when the oracle's fp64 theta is passed in) and
    rounded once to `out_dtype`, the precision the gradient buffer is handed
    over in."""
    sigma = problem.sigma if sigma is None else sigma
    dt = theta.dtype
    g = (theta - problem.theta_star.to(dt)).mul_(problem.h.to(dt))
    if noise is not None and sigma != 0.0:
        g.add_(noise.to(dt), alpha=sigma)
    return g.to(out_dtype)


def split_like(flat: torch.Tensor, layout: List[Tuple[str, int]], align_elems: int = 4) -> List[torch.Tensor]:
    """Views of `flat`, one per tensor of `layout`, each starting on a multiple
    of `align_elems` elements (so fp32 views stay 16-byte aligned)."""
    views, off = [], 0
    for _, n in layout:
        views.append(flat[off:off + n])
        off += -(-n // align_elems) * align_elems
    assert off <= flat.numel() + align_elems
    return views


def padded_numel(layout: List[Tuple[str, int]], align_elems: int = 4) -> int:
    return sum(-(-n // align_elems) * align_elems for _, n in layout)


# ---------------------------------------------------------------------------
# the same noisy quadratic for buffers too large to keep h, theta_star and the
# noise resident: everything is regenerated chunk by chunk from counters
# ---------------------------------------------------------------------------
class ChunkedQuadratic:
    """policy_problem() / surrogate-style data over a flat buffer of `numel`
    elements, produced in chunks of `chunk` elements.  Chunk c of h,
    theta_star, theta_0 comes from a generator seeded with (seed, c); chunk c of
    the noise of training step t from one seeded with (seed, t, c).  Any chunk
    can therefore be regenerated on its own, on the GPU for the engine or for a
    slice the oracle checks."""

    def __init__(self, numel: int, seed: int, sigma: float = 0.05, *, h_dist="loguniform", h_lo=1e-3, h_hi=1.0,
                 theta_std=0.02, chunk: int = 1 << 27, device="cuda"):
        self.numel, self.seed, self.sigma, self.chunk, self.device = numel, seed, sigma, chunk, device
        self.h_dist, self.h_lo, self.h_hi, self.theta_std = h_dist, h_lo, h_hi, theta_std

    def n_chunks(self) -> int:
        return -(-self.numel // self.chunk)

    def chunk_range(self, c: int) -> Tuple[int, int]:
        lo = c * self.chunk
        return lo, min(self.numel, lo + self.chunk)

    def chunk_problem(self, c: int) -> QuadraticProblem:
        lo, hi = self.chunk_range(c)
        return make_quadratic(hi - lo, self.seed * 7919 + 104729 * c + 1, h_dist=self.h_dist, h_lo=self.h_lo,
                              h_hi=self.h_hi, theta_std=self.theta_std, sigma=self.sigma, device=self.device)

    def chunk_noise(self, step: int, c: int) -> torch.Tensor:
        lo, hi = self.chunk_range(c)
        gen = _gen(self.device, (self.seed + 1) * 1_000_003 + step * 15_485_863 + c)
        return torch.randn(hi - lo, generator=gen, device=self.device, dtype=torch.float32)

    def init_theta(self, out: torch.Tensor) -> None:
        for c in range(self.n_chunks()):
            lo, hi = self.chunk_range(c)
            out[lo:hi].copy_(self.chunk_problem(c).theta_0)

    def grad(self, theta: torch.Tensor, step: int, out: torch.Tensor, sigma: float | None = None) -> None:
        """out <- h * (theta - theta_star) + sigma * xi_step, rounded to out.dtype."""
        for c in range(self.n_chunks()):
            lo, hi = self.chunk_range(c)
            p = self.chunk_problem(c)
            out[lo:hi].copy_(quadratic_grad(p, theta[lo:hi], self.chunk_noise(step, c), sigma, out_dtype=out.dtype))
