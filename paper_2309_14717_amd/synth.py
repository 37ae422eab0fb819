"""Seeded synthetic inputs for a QA-LoRA linear layer.

This module holds none of the method's arithmetic: it only draws random tensors
with the shapes and value distributions of the benchmark configurations (LLaMA
layer shapes, Gaussian weights of std 0.02, unit-variance activations with a few
outlier channels).  Both the CPU oracle's tests and the GPU path's tests take
their inputs from here, so the two sides see the same numbers.

Draw order is fixed: W, x, A, B, dy, then the outlier channel choice.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np
import torch


@dataclass(frozen=True)
class LayerConfig:
    name: str
    tokens: int
    d_in: int
    d_out: int
    bits: int = 4
    group: int = 32
    rank: int = 64
    s: float = 0.25
    seed: int = 0
    outlier_frac: float = 0.0   # fraction of input channels of x scaled by outlier_scale
    outlier_scale: float = 20.0
    w_std: float = 0.02
    ab_std: float = 0.02

    @property
    def groups(self) -> int:
        return self.d_in // self.group

    def scaled(self, **kw) -> "LayerConfig":
        return replace(self, **kw)


# The benchmark configurations (seed = configuration index - 1).
CONFIGS = {
    "c1": LayerConfig("c1", 64, 1024, 1024, 4, 32, 16, 2.0, seed=0),
    "c2": LayerConfig("c2", 4096, 4096, 4096, 4, 32, 64, 0.25, seed=1, outlier_frac=0.001),
    "c3_gate": LayerConfig("c3_gate", 4096, 4096, 11008, 4, 32, 64, 0.25, seed=2, outlier_frac=0.001),
    "c3_up": LayerConfig("c3_up", 4096, 4096, 11008, 4, 32, 64, 0.25, seed=12, outlier_frac=0.001),
    "c3_down": LayerConfig("c3_down", 4096, 11008, 4096, 4, 32, 64, 0.25, seed=22, outlier_frac=0.001),
    "c4": LayerConfig("c4", 2048, 5120, 13824, 4, 32, 64, 0.25, seed=3),
    "c5_up": LayerConfig("c5_up", 16, 8192, 22016, 4, 32, 64, 0.25, seed=4),
    "c5_down": LayerConfig("c5_down", 16, 22016, 8192, 4, 32, 64, 0.25, seed=14),
}


def bf16_round(a: torch.Tensor) -> torch.Tensor:
    """fp32 tensor holding values that are exactly representable in bfloat16."""
    return a.to(torch.bfloat16).to(torch.float32)


def make_inputs(cfg: LayerConfig, want=("W", "x", "A", "B", "dy")) -> dict:
    """Draw the tensors of one layer as fp32 numpy arrays.

    x and dy hold bf16-representable values (they are bf16 at the library boundary).
    Tensors not listed in ``want`` are still drawn (so the stream of random numbers,
    and therefore every other tensor, does not depend on ``want``) but not returned.
    """
    gen = torch.Generator(device="cpu").manual_seed(int(cfg.seed))
    out = {}

    def draw(name, shape, std, as_bf16=False):
        t = torch.randn(shape, generator=gen, dtype=torch.float32) * std
        if as_bf16:
            t = bf16_round(t)
        if name in want:
            out[name] = t
        return t

    draw("W", (cfg.d_in, cfg.d_out), cfg.w_std)
    x = draw("x", (cfg.tokens, cfg.d_in), 1.0)
    draw("A", (cfg.groups, max(cfg.rank, 1)), cfg.ab_std)
    draw("B", (max(cfg.rank, 1), cfg.d_out), cfg.ab_std)
    draw("dy", (cfg.tokens, cfg.d_out), 1.0, as_bf16=True)
    n_out = int(round(cfg.outlier_frac * cfg.d_in))
    if n_out > 0:
        idx = torch.randperm(cfg.d_in, generator=gen)[:n_out]
        x[:, idx] *= cfg.outlier_scale
        out["outlier_channels"] = idx
    if "x" in want:
        out["x"] = bf16_round(x)
    res = {}
    for k, v in out.items():
        res[k] = v.numpy() if isinstance(v, torch.Tensor) else v
    return res


def random_codes(cfg: LayerConfig):
    """Uniform random codes with Gaussian-derived alpha / beta, for cases that start
    from an already-quantized layer (any (codes, alpha, beta) triple is a valid input
    of forward / backward / merge)."""
    gen = torch.Generator(device="cpu").manual_seed(int(cfg.seed) + 1000)
    codes = torch.randint(0, 1 << cfg.bits, (cfg.d_in, cfg.d_out), generator=gen, dtype=torch.uint8)
    alpha = (torch.rand((cfg.groups, cfg.d_out), generator=gen) * 0.01 + 0.002).float()
    beta = (torch.randn((cfg.groups, cfg.d_out), generator=gen) * 0.01 - 0.04).float()
    return codes.numpy(), alpha.numpy(), beta.numpy()
