"""Seeded context lengths and allocator op scripts (pure data, no allocator logic).

A script is a list of tuples that any allocator front end can replay:
    ("extend", request, kind, new_len)        request's kind must hold tokens [0,new_len)
    ("share",  src, dst, kind, n_pages)       dst starts as a sharer of src's first pages
    ("free",   request)                       request finished: all its pages are freed
and, for low-level traces against alloc/ref/free directly,
    ("alloc", handle, kind, request) / ("ref", handle) / ("unref", handle)
where a handle is a trace-local name for the small page an "alloc" returns.
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import numpy as np

from .configs import CROSS, FULL, OPAQUE, WINDOW, ModelCfg

REQ_BASE = 100
DUMMY_BASE = 1_000_000


def request_id(b: int) -> int:
    return REQ_BASE + b


def sample_ctx(cfg: ModelCfg, seed: int) -> np.ndarray:
    """Tokens already cached per request before the decode step."""
    rng = np.random.default_rng([seed, 11])
    d = cfg.ctx
    if d.kind == "uniform":
        return rng.integers(d.lo, d.hi + 1, size=cfg.batch).astype(np.int64)
    if d.kind == "lognormal":
        x = np.exp(rng.normal(math.log(d.median), d.sigma, size=cfg.batch))
        return np.clip(np.rint(x), d.lo, d.hi).astype(np.int64)
    raise ValueError(d.kind)


def sharers(cfg: ModelCfg, ctx: np.ndarray, seed: int) -> List[int]:
    """Batch indices of the one prefix-sharing group, leader first (may be empty)."""
    if cfg.share_fraction <= 0:
        return []
    rng = np.random.default_rng([seed, 13])
    eligible = [b for b in range(cfg.batch) if ctx[b] >= cfg.share_tokens]
    n = min(len(eligible), int(round(cfg.share_fraction * cfg.batch)))
    if n < 2:
        return []
    return [int(b) for b in rng.permutation(eligible)[:n]]


def _first_touch(cfg: ModelCfg, ops: list, rid: int) -> None:
    for k, kind in enumerate(cfg.kinds):
        if kind.type == CROSS:
            ops.append(("extend", rid, k, cfg.cross_len))
        elif kind.type == OPAQUE:
            ops.append(("extend", rid, k, 1))


def build_script(cfg: ModelCfg, ctx: Sequence[int], seed: int) -> List[tuple]:
    """Ops that bring every request to ctx[b] cached tokens, interleaved.

    Requests grow by cfg.build_chunk tokens per round in a seeded random order
    (so their pages interleave in the pool, as Sec. 4.3 describes for real
    serving); short-lived dummy requests grow alongside and are freed at the
    end in random order, leaving holes.
    """
    rng = np.random.default_rng([seed, 17])
    ops: List[tuple] = []
    token_kinds = [k for k, kd in enumerate(cfg.kinds) if kd.type in (FULL, WINDOW)]
    target = {request_id(b): int(ctx[b]) for b in range(cfg.batch)}
    for i in range(cfg.n_dummy):
        target[DUMMY_BASE + i] = int(rng.integers(cfg.dummy_ctx[0], cfg.dummy_ctx[1] + 1))
    cur = {rid: 0 for rid in target}
    touched = set()

    group = sharers(cfg, ctx, seed)
    if group:
        lead = request_id(group[0])
        _first_touch(cfg, ops, lead)
        touched.add(lead)
        for k in token_kinds:
            ops.append(("extend", lead, k, cfg.share_tokens))
        cur[lead] = cfg.share_tokens
        n_pages = {k: cfg.share_tokens // cfg.kinds[k].tokens_per_page for k in token_kinds}
        for b in group[1:]:
            rid = request_id(b)
            _first_touch(cfg, ops, rid)
            touched.add(rid)
            for k in token_kinds:
                if cfg.kinds[k].type == FULL:
                    ops.append(("share", lead, rid, k, n_pages[k]))
                else:
                    ops.append(("extend", rid, k, cfg.share_tokens))
            cur[rid] = cfg.share_tokens

    rids = sorted(target)
    while True:
        todo = [rid for rid in rids if cur[rid] < target[rid]]
        if not todo:
            break
        for j in rng.permutation(len(todo)):
            rid = todo[int(j)]
            if rid not in touched:
                _first_touch(cfg, ops, rid)
                touched.add(rid)
            new_len = min(target[rid], cur[rid] + cfg.build_chunk)
            for k in token_kinds:
                ops.append(("extend", rid, k, new_len))
            cur[rid] = new_len
    dummies = [rid for rid in rids if rid >= DUMMY_BASE]
    for j in rng.permutation(len(dummies)):
        ops.append(("free", dummies[int(j)]))
    return ops


def step_script(cfg: ModelCfg, ctx: Sequence[int]) -> List[tuple]:
    """Host side of one decode step: room for token ctx[b] (length becomes ctx[b]+1)."""
    ops = []
    for b in range(cfg.batch):
        for k, kd in enumerate(cfg.kinds):
            if kd.type in (FULL, WINDOW):
                ops.append(("extend", request_id(b), k, int(ctx[b]) + 1))
    return ops


def finish_script(cfg: ModelCfg, seed: int) -> List[tuple]:
    rng = np.random.default_rng([seed, 19])
    return [("free", request_id(int(b))) for b in rng.permutation(cfg.batch)]


def run_script(ops: Sequence[tuple], front) -> None:
    """front: any object with extend / share_prefix / free_request."""
    for op in ops:
        if op[0] == "extend":
            front.extend(op[1], op[2], op[3])
        elif op[0] == "share":
            front.share_prefix(op[1], op[2], op[3], op[4])
        elif op[0] == "free":
            front.free_request(op[1])
        else:
            raise ValueError(op)


def pool_large_pages_needed(cfg: ModelCfg, ctx: Sequence[int], large_bytes: int,
                            headroom: float = 1.10) -> int:
    """Upper bound on large pages the build + one step can hold live, with headroom."""
    total = 0
    for kd in cfg.kinds:
        S = kd.small_page_bytes
        r = large_bytes // S
        pages = 0
        T = kd.tokens_per_page
        for b in range(cfg.batch):
            if kd.type == FULL:
                n = -(-(int(ctx[b]) + 1) // T)
            elif kd.type == WINDOW:
                n = min(-(-(int(ctx[b]) + 1) // T), (kd.window + cfg.build_chunk) // T + 2)
            elif kd.type == CROSS:
                n = -(-cfg.cross_len // T)
            else:
                n = 1
            pages += -(-n // r) * r          # whole large pages per request (Sec. 4.3)
        pages += cfg.n_dummy * (-(-cfg.dummy_ctx[1] // T) + r)
        total += -(-pages // r)
    return int(total * headroom) + 8


def lowlevel_trace(n_kinds: int, n_requests: int, n_ops: int, seed: int,
                   p_free: float = 0.35, p_ref: float = 0.05,
                   burst_free: float = 0.02) -> List[tuple]:
    """Random alloc / ref / unref trace; every handle ends up fully released."""
    rng = np.random.default_rng([seed, 23])
    ops: List[tuple] = []
    live: List[Tuple[int, int]] = []       # (handle, request), one entry per reference
    nxt = 0
    for _ in range(n_ops):
        u = rng.random()
        if live and u < burst_free:
            # a request finishes: all its references go at once (Sec. 4.3)
            req = live[int(rng.integers(len(live)))][1]
            for h, r in [e for e in live if e[1] == req]:
                ops.append(("unref", h))
            live = [e for e in live if e[1] != req]
        elif live and u < burst_free + p_free:
            j = int(rng.integers(len(live)))
            ops.append(("unref", live[j][0]))
            live.pop(j)
        elif live and u < burst_free + p_free + p_ref:
            j = int(rng.integers(len(live)))
            ops.append(("ref", live[j][0]))
            live.append(live[j])
        else:
            k = int(rng.integers(n_kinds))
            req = int(rng.integers(n_requests)) + 1
            ops.append(("alloc", nxt, k, req))
            live.append((nxt, req))
            nxt += 1
    for j in rng.permutation(len(live)):
        ops.append(("unref", live[int(j)][0]))
    return ops
