"""Shapes of the five synthetic workloads (no arithmetic of the method here).

Each config stands in for one of the paper's evaluated model families
(Table 1, Sec. 7.1) by its *shape* only: layer mix, head counts, head
dimension, window, context-length range.  No dataset item or weight is used.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

ELEM_BYTES = {"f32": 4, "bf16": 2}

FULL, WINDOW, CROSS, OPAQUE = "full", "window", "cross", "opaque"


@dataclass
class KindCfg:
    name: str
    type: str                     # full | window | cross | opaque
    dtype: str = "bf16"           # f32 | bf16
    n_layers: int = 1
    n_q_heads: int = 0
    n_kv_heads: int = 0
    head_dim: int = 0
    tokens_per_page: int = 16
    window: int = 0
    opaque_page_bytes: int = 0    # OPAQUE kinds only: bytes of one small page

    @property
    def elem_bytes(self) -> int:
        return ELEM_BYTES[self.dtype]

    @property
    def slice_bytes(self) -> int:
        """One layer's K+V for one page of tokens."""
        if self.type == OPAQUE:
            return self.opaque_page_bytes // max(1, self.n_layers)
        return 2 * self.n_kv_heads * self.tokens_per_page * self.head_dim * self.elem_bytes

    @property
    def small_page_bytes(self) -> int:
        """All layers of the kind for one page of tokens (page-layer partition, Sec. 4.2)."""
        if self.type == OPAQUE:
            return self.opaque_page_bytes
        return self.n_layers * self.slice_bytes

    @property
    def bytes_per_token_per_layer(self) -> int:
        return 2 * self.n_kv_heads * self.head_dim * self.elem_bytes


@dataclass
class LengthDist:
    kind: str                     # "uniform" | "lognormal"
    lo: int
    hi: int
    median: float = 0.0
    sigma: float = 1.0            # ln-space sigma for lognormal


@dataclass
class ModelCfg:
    name: str
    kinds: List[KindCfg]
    batch: int
    ctx: LengthDist               # tokens already cached before the decode step
    cross_len: int = 0            # fixed encoder length for CROSS kinds
    value_sigma: float = 1.0
    pool_large_pages: Optional[int] = None   # None: sized from the workload with headroom
    build_chunk: int = 256        # tokens per request per round while contexts are built
    n_dummy: int = 0              # short-lived requests interleaved with the real ones
    dummy_ctx: Tuple[int, int] = (1, 96)
    share_fraction: float = 0.0   # fraction of requests sharing a prefix (one group)
    share_tokens: int = 0
    notes: str = ""


def tiny() -> ModelCfg:
    return ModelCfg(
        name="tiny",
        kinds=[
            KindCfg("A_full", FULL, "f32", 1, 4, 2, 64, 16),
            KindCfg("B_window32", WINDOW, "f32", 1, 4, 2, 128, 16, window=32),
        ],
        batch=4, ctx=LengthDist("uniform", 1, 256),
        pool_large_pages=64, build_chunk=16, n_dummy=2, dummy_ctx=(1, 96),
    )


def mini_bf16() -> ModelCfg:
    """A seconds-sized bf16 case for smoke checks: one full-attention kind with 256-element rows
    and 2 query heads per KV head, one sliding-window kind with 128-element rows and 4."""
    return ModelCfg(
        name="mini_bf16",
        kinds=[
            KindCfg("full", FULL, "bf16", 2, 4, 2, 256, 16),
            KindCfg("window96", WINDOW, "bf16", 3, 8, 2, 128, 16, window=96),
        ],
        batch=5, ctx=LengthDist("uniform", 1, 700), value_sigma=0.5,
        build_chunk=32, n_dummy=2, dummy_ctx=(1, 96),
    )


def gemma2_9b() -> ModelCfg:
    return ModelCfg(
        name="gemma2_9b",
        kinds=[
            KindCfg("full", FULL, "bf16", 21, 16, 8, 256, 16),
            KindCfg("window4096", WINDOW, "bf16", 21, 16, 8, 256, 16, window=4096),
        ],
        batch=64, ctx=LengthDist("uniform", 2048, 8192), value_sigma=0.5,
        build_chunk=512,
    )


def llama32_vision_11b() -> ModelCfg:
    return ModelCfg(
        name="llama32_vision_11b",
        kinds=[
            KindCfg("self", FULL, "bf16", 32, 32, 8, 128, 16),
            KindCfg("cross", CROSS, "bf16", 8, 32, 8, 128, 16),
        ],
        batch=32, ctx=LengthDist("uniform", 512, 4096), cross_len=1601 * 4,
        build_chunk=512,
    )


def jamba_like(literal: bool = False) -> ModelCfg:
    """literal=True: one small page per layer (64 KiB / 512 KiB, LCM 512 KiB)."""
    n_attn, n_mamba = (1, 1) if literal else (4, 28)
    return ModelCfg(
        name="jamba_like_literal" if literal else "jamba_like",
        kinds=[
            KindCfg("attn", FULL, "bf16", n_attn, 32, 8, 128, 16),
            KindCfg("mamba_state", OPAQUE, "f32", n_mamba, tokens_per_page=1,
                    opaque_page_bytes=n_mamba * 8192 * 16 * 4),
        ],
        batch=128, ctx=LengthDist("lognormal", 128, 32768, median=2048.0, sigma=1.0),
        build_chunk=512,
    )


def long_5to1() -> ModelCfg:
    return ModelCfg(
        name="long_5to1",
        kinds=[
            KindCfg("window1024", WINDOW, "bf16", 40, 32, 8, 128, 16, window=1024),
            KindCfg("full", FULL, "bf16", 8, 32, 8, 128, 16),
        ],
        batch=32, ctx=LengthDist("lognormal", 1024, 131072, median=16384.0, sigma=1.0),
        value_sigma=0.5, build_chunk=2048, share_fraction=0.25, share_tokens=4096,
    )


def short_b1024() -> ModelCfg:
    """Many short requests: the regime a larger decode batch (what the paper's memory savings buy,
    Sec. 7.3) pushes the kernel into.  A homogeneous Llama-3.1-8B-shaped model (32 full-attention
    layers, 32 query and 8 KV heads of 128 elements; Table 1 lists Llama 3.1 as the homogeneous
    control), batch 1024, 100 to 600 cached tokens per request."""
    return ModelCfg(
        name="short_b1024",
        kinds=[KindCfg("full", FULL, "bf16", 32, 32, 8, 128, 16)],
        batch=1024, ctx=LengthDist("uniform", 100, 600),
        build_chunk=128,
    )


def jamba_like_literal() -> ModelCfg:
    return jamba_like(literal=True)


ALL = {
    "tiny": tiny,
    "gemma2_9b": gemma2_9b,
    "llama32_vision_11b": llama32_vision_11b,
    "jamba_like": jamba_like,
    "long_5to1": long_5to1,
    "short_b1024": short_b1024,
    "jamba_like_literal": jamba_like_literal,
}


def layer_schedule(cfg: ModelCfg):
    """Model order of the attention layers as (kind index, layer within kind).

    Kinds are interleaved in proportion to their layer counts (alternating for the
    Gemma-2 shape, every fifth layer cross-attention for the Llama-3.2-Vision shape).
    """
    att = [(i, k) for i, k in enumerate(cfg.kinds) if k.type != OPAQUE]
    total = sum(k.n_layers for _, k in att)
    done = {i: 0 for i, _ in att}
    out = []
    for step in range(total):
        # pick the kind that is furthest behind its share
        i, k = min(att, key=lambda ik: ((done[ik[0]] + 1) / ik[1].n_layers, -ik[1].n_layers)
                   if done[ik[0]] < ik[1].n_layers else (float("inf"), 0))
        out.append((i, done[i]))
        done[i] += 1
    return out
