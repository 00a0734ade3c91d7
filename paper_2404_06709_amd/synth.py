"""Seeded synthetic inputs for the CQIL hot path.

This module holds none of the method's arithmetic: it only draws random tensors with the
shapes and value distributions of the workloads (LLaMA-1 layer shapes; weights N(0, 0.02),
norm gains 1.0 (optionally jittered for tests), hidden states and KV-cache fill N(0, 1)) and
converts between torch and numpy views.  Both the HIP path's tests and the CPU oracle's tests
draw their inputs here so they see bit-identical data.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List

import numpy as np
import torch


@dataclass(frozen=True)
class Shape:
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int


SHAPES: Dict[str, Shape] = {
    "tiny": Shape(256, 4, 64, 688),
    "7b": Shape(4096, 32, 128, 11008),
    "13b": Shape(5120, 40, 128, 13824),
    "33b": Shape(6656, 52, 128, 17920),
}

LAYER_KEYS = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "g_attn", "g_ffn")


def generator(seed: int, device: str = "cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def normal(shape, std: float, dtype: torch.dtype, gen: torch.Generator) -> torch.Tensor:
    """N(0, std) drawn in fp32 on the generator's device, then rounded to ``dtype``."""
    t = torch.empty(shape, dtype=torch.float32, device=gen.device)
    t.normal_(0.0, std, generator=gen)
    return t.to(dtype)


def make_layer(shape: Shape, dtype: torch.dtype, gen: torch.Generator, w_std: float = 0.02,
               gain_jitter: float = 0.0) -> Dict[str, torch.Tensor]:
    dm, f = shape.d_model, shape.d_ffn
    L = {
        "wq": normal((dm, dm), w_std, dtype, gen),
        "wk": normal((dm, dm), w_std, dtype, gen),
        "wv": normal((dm, dm), w_std, dtype, gen),
        "wo": normal((dm, dm), w_std, dtype, gen),
        "wgate": normal((f, dm), w_std, dtype, gen),
        "wup": normal((f, dm), w_std, dtype, gen),
        "wdown": normal((dm, f), w_std, dtype, gen),
    }
    for k in ("g_attn", "g_ffn"):
        g = torch.ones(dm, dtype=torch.float32, device=gen.device)
        if gain_jitter:
            g = g + normal((dm,), gain_jitter, torch.float32, gen)
        L[k] = g.to(dtype)
    return L


def make_layers(n: int, shape: Shape, dtype: torch.dtype, seed: int, w_std: float = 0.02,
                gain_jitter: float = 0.0, device: str = "cpu") -> List[Dict[str, torch.Tensor]]:
    gen = generator(seed, device)
    return [make_layer(shape, dtype, gen, w_std, gain_jitter) for _ in range(n)]


def to_numpy(t: torch.Tensor) -> np.ndarray:
    """fp32 -> float32 array; bf16 -> uint16 array of the same bit patterns; ints unchanged."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def layer_to_numpy(layer: Dict[str, torch.Tensor]) -> Dict[str, np.ndarray]:
    return {k: to_numpy(layer[k]) for k in LAYER_KEYS}


def widen(t: torch.Tensor) -> np.ndarray:
    """Exact float64 copy of an fp32 / bf16 tensor."""
    return t.detach().cpu().to(torch.float64).numpy()


def kv_lengths(batch: int, lo: int, hi: int, seed: int) -> np.ndarray:
    """Per-sequence cache lengths drawn uniformly from [lo, hi]."""
    gen = generator(seed)
    return torch.randint(lo, hi + 1, (batch,), generator=gen).to(torch.int32).numpy()
