"""Seeded N(0, sigma) values rounded to the pool's storage type (torch CPU tensors)."""
from __future__ import annotations

import torch

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def _gen(seed: int, *stream: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    s = seed & 0x7FFFFFFF
    for x in stream:
        s = (s * 1000003 + (x & 0x7FFFFFFF) + 12345) % (2 ** 61 - 1)
    g.manual_seed(s)
    return g


def normal(shape, dtype: str, sigma: float, seed: int, *stream: int) -> torch.Tensor:
    """fp32 normal draws scaled by sigma, then rounded (RNE) to the storage type."""
    x = torch.randn(*shape, generator=_gen(seed, *stream), dtype=torch.float32) * sigma
    return x.to(TORCH_DTYPE[dtype])


def kv_for_request(kind, layer: int, request: int, length: int, sigma: float, seed: int):
    """Contiguous K, V [H_kv, length, D] of one request in one layer."""
    shape = (kind.n_kv_heads, length, kind.head_dim)
    K = normal(shape, kind.dtype, sigma, seed, 1, layer, request)
    V = normal(shape, kind.dtype, sigma, seed, 2, layer, request)
    return K, V


def q_for_layer(kind, layer: int, batch: int, sigma: float, seed: int) -> torch.Tensor:
    return normal((batch, kind.n_q_heads, kind.head_dim), kind.dtype, sigma, seed, 3, layer)
