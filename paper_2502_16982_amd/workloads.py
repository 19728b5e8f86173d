"""Seeded synthetic inputs for the Muon step: shapes and value distributions only.

This module holds none of the method's arithmetic.  It serves both the HIP
library's tests/bench and the CPU oracle's tests, so that both sides see the
same buffers.

The paper measures the optimizer on no public benchmark; the workloads below
take their *shapes* from its model families (square attention projections,
[H, 4H] / SwiGLU MLP matrices, a 64-expert MoE bank) and their value
distributions from the benchmark definition: W ~ N(0, 0.02^2) (N(0,1) for the
small fp32 case), G ~ N(0, (1e-3)^2) (N(0,1) for the small fp32 case), momentum
zero-initialised, optionally 1 % of gradient entries multiplied by 100.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import torch


@dataclass(frozen=True)
class Hyper:
    lr: float = 0.02
    weight_decay: float = 0.1
    momentum: float = 0.95
    a: float = 3.4445
    b: float = -4.7750
    c: float = 2.0315
    rms_scale: float = 0.2
    eps: float = 1e-7
    ns_steps: int = 5
    nesterov: bool = True


@dataclass(frozen=True)
class Workload:
    name: str
    shapes: Tuple[Tuple[int, int], ...]      # (A, B) per matrix, in list order
    w_dtype: torch.dtype
    g_dtype: torch.dtype
    ns_dtype: str                             # "bf16", "f32", "bf16x2" or "bf16x3"
    w_std: float
    g_std: float
    outlier_frac: float = 0.0
    outlier_mult: float = 1.0
    seed_base: int = 0
    hyper: Hyper = field(default_factory=Hyper)

    @property
    def n_elements(self) -> int:
        return sum(a * b for a, b in self.shapes)

    def ns_flops(self, ns_steps: int | None = None) -> int:
        """Nominal Newton-Schulz flop count: N * (4 m^2 n + 2 m^3) per matrix, m <= n."""
        n_it = self.hyper.ns_steps if ns_steps is None else ns_steps
        tot = 0
        for a, b in self.shapes:
            m, n = min(a, b), max(a, b)
            tot += n_it * (4 * m * m * n + 2 * m * m * m)
        return tot


def _dense_transformer(layers: int, width: int, ffn: int) -> Tuple[Tuple[int, int], ...]:
    per_layer = [(width, width)] * 4 + [(width, ffn)] * 2 + [(ffn, width)]
    return tuple(per_layer * layers)


def _moe_bank(experts: int, hidden: int, inter: int) -> Tuple[Tuple[int, int], ...]:
    per_expert = [(hidden, inter), (hidden, inter), (inter, hidden)]
    return tuple(per_expert * experts)


def workload(name: str) -> Workload:
    """The five benchmark configurations, by name."""
    bf16, f32 = torch.bfloat16, torch.float32
    if name == "single_128x256_f32":
        return Workload(name, ((128, 256),), f32, f32, "f32", 1.0, 1.0, seed_base=0)
    if name == "dense12_w1024":
        return Workload(name, _dense_transformer(12, 1024, 4096), bf16, bf16, "bf16", 0.02, 1e-3, seed_base=2000)
    if name == "block_w4096":
        shapes = ((4096, 4096),) * 4 + ((4096, 11008),) * 2 + ((11008, 4096),)
        return Workload(name, shapes, bf16, bf16, "bf16", 0.02, 1e-3, 0.01, 100.0, seed_base=3000)
    if name == "moe_bank_66x2048x1408":
        return Workload(name, _moe_bank(66, 2048, 1408), bf16, bf16, "bf16", 0.02, 1e-3, seed_base=4000)
    if name == "moe27_w2048":
        per_layer = _moe_bank(66, 2048, 1408) + ((2048, 2048),) * 4
        return Workload(name, tuple(per_layer * 27), bf16, bf16, "bf16", 0.02, 1e-3, seed_base=5000)
    raise KeyError(name)


WORKLOAD_NAMES = ("single_128x256_f32", "dense12_w1024", "block_w4096", "moe_bank_66x2048x1408", "moe27_w2048")


def custom(name: str, shapes, *, w_dtype=torch.bfloat16, g_dtype=torch.bfloat16, ns_dtype="bf16",
           w_std=0.02, g_std=1e-3, outlier_frac=0.0, outlier_mult=1.0, seed_base=0, hyper=None) -> Workload:
    return Workload(name, tuple((int(a), int(b)) for a, b in shapes), w_dtype, g_dtype, ns_dtype, w_std, g_std,
                    outlier_frac, outlier_mult, seed_base, hyper or Hyper())


def make_matrix(wl: Workload, index: int, device="cpu"):
    """(W, G, M0) for matrix ``index`` of a workload, generated on ``device`` from seed_base + index."""
    a, b = wl.shapes[index]
    gen = torch.Generator(device=device)
    gen.manual_seed(wl.seed_base + index)
    w = torch.empty((a, b), dtype=torch.float32, device=device).normal_(0.0, wl.w_std, generator=gen)
    g = torch.empty((a, b), dtype=torch.float32, device=device).normal_(0.0, wl.g_std, generator=gen)
    if wl.outlier_frac > 0.0:
        mask = torch.empty((a, b), dtype=torch.float32, device=device).uniform_(0.0, 1.0, generator=gen) < wl.outlier_frac
        g = torch.where(mask, g * wl.outlier_mult, g)
    m = torch.zeros((a, b), dtype=torch.float32, device=device)
    return w.to(wl.w_dtype).contiguous(), g.to(wl.g_dtype).contiguous(), m


def make_gradient(wl: Workload, index: int, step: int, device="cpu"):
    """A fresh gradient for a later step (same distribution, different seed)."""
    a, b = wl.shapes[index]
    gen = torch.Generator(device=device)
    gen.manual_seed(wl.seed_base + index + 7919 * (step + 1))
    g = torch.empty((a, b), dtype=torch.float32, device=device).normal_(0.0, wl.g_std, generator=gen)
    if wl.outlier_frac > 0.0:
        mask = torch.empty((a, b), dtype=torch.float32, device=device).uniform_(0.0, 1.0, generator=gen) < wl.outlier_frac
        g = torch.where(mask, g * wl.outlier_mult, g)
    return g.to(wl.g_dtype).contiguous()


def make_all(wl: Workload, device="cpu") -> List[tuple]:
    return [make_matrix(wl, i, device) for i in range(len(wl.shapes))]
