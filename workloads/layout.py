"""The harness's own statement of the pool's address map, in torch indexing.

Small page `sid` of a kind starts sid * small_page_bytes from the pool base
(Sec. 4.1 last paragraph, Sec. 4.2).  Inside it the layers of the kind follow
one another (page-layer partition, Sec. 4.2); a layer's slice is laid out
[H_kv][K|V][T][D].  Written independently of the library so that scatter /
gather through it cross-checks the kernels' addressing.
"""
from __future__ import annotations

from typing import Sequence

import torch

from .values import TORCH_DTYPE


def _slice_view(pool_u8: torch.Tensor, kind, sid: int, layer: int) -> torch.Tensor:
    begin = sid * kind.small_page_bytes + layer * kind.slice_bytes
    raw = pool_u8[begin:begin + kind.slice_bytes]
    return raw.view(TORCH_DTYPE[kind.dtype]).view(
        kind.n_kv_heads, 2, kind.tokens_per_page, kind.head_dim)


def scatter_request(pool_u8: torch.Tensor, kind, layer: int, row: Sequence[int],
                    K: torch.Tensor, V: torch.Tensor, length: int) -> None:
    """Write tokens [0, length) of contiguous K, V [H_kv, >=length, D] into resident pages."""
    T = kind.tokens_per_page
    for p in range(-(-length // T)):
        sid = int(row[p])
        if sid < 0:
            continue
        n = min(T, length - p * T)
        view = _slice_view(pool_u8, kind, sid, layer)
        view[:, 0, :n, :] = K[:, p * T:p * T + n, :].to(view.device)
        view[:, 1, :n, :] = V[:, p * T:p * T + n, :].to(view.device)


def gather_request(pool_u8: torch.Tensor, kind, layer: int, row: Sequence[int],
                   length: int):
    """Contiguous K, V [H_kv, length, D] (CPU); tokens of non-resident pages are NaN."""
    T = kind.tokens_per_page
    dt = TORCH_DTYPE[kind.dtype]
    K = torch.full((kind.n_kv_heads, length, kind.head_dim), float("nan"), dtype=dt)
    V = torch.full_like(K, float("nan"))
    n_pages = -(-length // T)
    ids = torch.as_tensor([int(row[p]) for p in range(n_pages)], dtype=torch.int64)
    res = torch.nonzero(ids >= 0).flatten()
    if res.numel() == 0:
        return K, V
    per = kind.slice_bytes // kind.elem_bytes
    base = (ids[res] * kind.small_page_bytes + layer * kind.slice_bytes) // kind.elem_bytes
    typed = pool_u8.view(dt)
    idx = base.to(pool_u8.device)[:, None] + torch.arange(per, device=pool_u8.device)[None, :]
    blocks = typed[idx].view(-1, kind.n_kv_heads, 2, T, kind.head_dim).cpu()
    for j, p in enumerate(res.tolist()):
        n = min(T, length - p * T)
        K[:, p * T:p * T + n, :] = blocks[j, :, 0, :n, :]
        V[:, p * T:p * T + n, :] = blocks[j, :, 1, :n, :]
    return K, V


def fill_slice(pool_u8: torch.Tensor, kind, sid: int, layer: int, value: float) -> None:
    _slice_view(pool_u8, kind, sid, layer).fill_(value)
