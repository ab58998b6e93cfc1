"""Seeded synthetic workloads for decayed causal linear attention.

This module only draws inputs.  It holds none of the operator's arithmetic and
imports neither the HIP binding nor the CPU oracle, so both sides of a parity
test can be fed from it.

The paper's single-layer benchmark draws random tensors (Listing 2 uses
``torch.randn`` for B, C and V and a per-head ``gamma`` of shape (heads, 1));
its end-to-end runs use LongBench prompts, which are not available here and are
not needed: the operator's cost does not depend on the values.  Seeded Gaussian
tensors of the stated shapes stand in for them.

Recipe (the same for every configuration):
  * ``torch.Generator(device="cpu").manual_seed(seed)``;
  * draw fp32 ``q``, then ``k``, then ``v`` with ``torch.randn`` and multiply
    each by ``d ** -0.5`` (the operator itself applies no 1/sqrt(d), Section 2);
  * cast to the storage dtype (bf16 configurations round once, here);
  * per-head ``gamma`` is evaluated in fp64 and rounded to fp32 once.
For the decode workload the state is drawn first (sigma = 0.1), then q, k, v of
every step in step order.
"""
from __future__ import annotations

import dataclasses
from typing import Iterator, Optional, Tuple

import numpy as np
import torch


@dataclasses.dataclass(frozen=True)
class ForwardConfig:
    name: str
    B: int
    H: int
    N: int
    d: int
    dtype: str  # "f32" | "bf16"
    seed: int
    gamma_kind: str  # "scalar:<v>" | "pow2:<lo>:<hi>" (1 - 2**-(lo + h*(hi-lo)/(H-1)))

    @property
    def tokens(self) -> int:
        return self.B * self.N


@dataclasses.dataclass(frozen=True)
class DecodeConfig:
    name: str
    B: int
    H: int
    d: int
    steps: int
    seed: int
    gamma_kind: str
    state_sigma: float = 0.1
    dtype: str = "bf16"


# The five configurations of the benchmark definition.
CONFIG1 = ForwardConfig("cfg1_tiny_f32", 1, 1, 256, 64, "f32", 0, "scalar:0.9")
CONFIG2 = ForwardConfig("cfg2_small_f32", 2, 8, 2048, 64, "f32", 1, "pow2:5:12")
CONFIG3 = ForwardConfig("cfg3_mid_bf16", 4, 16, 4096, 128, "bf16", 2, "pow2:5:8")
CONFIG4 = ForwardConfig("cfg4_long_bf16", 1, 32, 32768, 128, "bf16", 3, "pow2:5:10")
CONFIG5 = DecodeConfig("cfg5_decode", 64, 32, 128, 256, 4, "pow2:5:10")

FORWARD_CONFIGS = {c.name: c for c in (CONFIG1, CONFIG2, CONFIG3, CONFIG4)}


def make_gamma(kind: str, H: int) -> torch.Tensor:
    """Per-head decay factors, fp32, shape [H].

    ``scalar:v`` repeats v.  ``pow2:lo:hi`` gives 1 - 2**-(lo + h*(hi-lo)/(H-1))
    for h = 0..H-1 (config 2: exponents 5..12 in steps of 1; config 3: 5..8;
    configs 4 and 5: 5..10), evaluated in fp64 and rounded to fp32 once.
    """
    parts = kind.split(":")
    if parts[0] == "scalar":
        g = np.full(H, float(parts[1]), dtype=np.float64)
    elif parts[0] == "pow2":
        lo, hi = float(parts[1]), float(parts[2])
        h = np.arange(H, dtype=np.float64)
        step = (hi - lo) / (H - 1) if H > 1 else 0.0
        g = 1.0 - np.exp2(-(lo + h * step))
    else:
        raise ValueError(f"unknown gamma kind {kind!r}")
    return torch.from_numpy(g.astype(np.float32))


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[name]


def draw_qkv(shape: Tuple[int, ...], d: int, dtype: str, gen: torch.Generator):
    """q, k, v ~ N(0,1)/sqrt(d), drawn in fp32 in that order, then cast."""
    scale = float(d) ** -0.5
    out = []
    for _ in range(3):
        x = torch.randn(shape, generator=gen, dtype=torch.float32)
        x.mul_(scale)
        out.append(x.to(torch_dtype(dtype)))
    return tuple(out)


def make_forward_inputs(cfg: ForwardConfig):
    """Returns (q, k, v, gamma) as CPU tensors; q, k, v are [B, H, N, d]."""
    gen = torch.Generator(device="cpu").manual_seed(cfg.seed)
    q, k, v = draw_qkv((cfg.B, cfg.H, cfg.N, cfg.d), cfg.d, cfg.dtype, gen)
    return q, k, v, make_gamma(cfg.gamma_kind, cfg.H)


def make_custom_forward_inputs(B: int, H: int, N: int, d: int, dtype: str, seed: int,
                               gamma: Optional[torch.Tensor] = None):
    """Same recipe at an arbitrary shape (ragged-tail and edge-case tests)."""
    gen = torch.Generator(device="cpu").manual_seed(seed)
    q, k, v = draw_qkv((B, H, N, d), d, dtype, gen)
    if gamma is None:
        gamma = make_gamma("pow2:3:9", H) if H > 1 else make_gamma("scalar:0.9", 1)
    return q, k, v, gamma.to(torch.float32)


def make_rd_forward_inputs(B: int, H: int, N: int, r: int, dv: int, dtype: str, seed: int,
                           gamma: Optional[torch.Tensor] = None):
    """Rank r different from the value width dv: q, k ~ N(0,1)/sqrt(r) [B,H,N,r], v ~ N(0,1)/sqrt(dv) [B,H,N,dv]."""
    gen = torch.Generator(device="cpu").manual_seed(seed)
    q = (torch.randn((B, H, N, r), generator=gen, dtype=torch.float32) * float(r) ** -0.5).to(torch_dtype(dtype))
    k = (torch.randn((B, H, N, r), generator=gen, dtype=torch.float32) * float(r) ** -0.5).to(torch_dtype(dtype))
    v = (torch.randn((B, H, N, dv), generator=gen, dtype=torch.float32) * float(dv) ** -0.5).to(torch_dtype(dtype))
    if gamma is None:
        gamma = make_gamma("pow2:3:9", H) if H > 1 else make_gamma("scalar:0.9", 1)
    return q, k, v, gamma.to(torch.float32)


def make_decode_state(cfg: DecodeConfig, gen: torch.Generator) -> torch.Tensor:
    """Initial state S[B, H, d, d] fp32 ~ N(0, sigma^2) (variance 0.01)."""
    s = torch.randn((cfg.B, cfg.H, cfg.d, cfg.d), generator=gen, dtype=torch.float32)
    return s.mul_(cfg.state_sigma)


def decode_stream(cfg: DecodeConfig) -> Tuple[torch.Tensor, torch.Tensor, Iterator]:
    """Returns (state0, gamma, iterator over per-step (q, k, v) each [B, H, d])."""
    gen = torch.Generator(device="cpu").manual_seed(cfg.seed)
    state0 = make_decode_state(cfg, gen)
    gamma = make_gamma(cfg.gamma_kind, cfg.H)

    def steps():
        for _ in range(cfg.steps):
            yield draw_qkv((cfg.B, cfg.H, cfg.d), cfg.d, cfg.dtype, gen)

    return state0, gamma, steps()


def to_f64(x: torch.Tensor) -> np.ndarray:
    """Exact widening of the stored values (bf16 or fp32) to a float64 array."""
    return x.to(torch.float64).contiguous().numpy()
