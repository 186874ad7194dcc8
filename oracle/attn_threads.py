"""A second CPU baseline for the benchmark's report: the same single-token decode attention in
fp32 with one task per (request, KV head) on a thread pool.

TEST INFRASTRUCTURE ONLY (see the package docstring), and not the parity oracle: attn.py stays
the reference every result is checked against.  This variant exists so that the CPU figure in the
benchmark's report is not only that of a deliberately plain fp64 loop: the definition is the
same (Sec. 4.2: attention "as usual" over the visible tokens; window of Sec. 5.1), computed in
the storage-friendly precision with the G query heads of a KV head sharing one pass over its
K and V, which is what a tuned CPU implementation would also do.  Pinned against attn.py in
tests/test_oracle_attn.py.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import List, Sequence

import numpy as np

from .attn import visible_range


def _one_kv_head(q_group: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float) -> np.ndarray:
    """q_group [G, D], K, V [n_vis, D] fp32 -> [G, D] fp32."""
    s = (K @ q_group.T) * np.float32(scale)            # [n_vis, G]
    s -= s.max(axis=0, keepdims=True)
    e = np.exp(s, out=s)
    return (e.T @ V) / e.sum(axis=0)[:, None]


def decode_attention_threads(q: np.ndarray, Ks: Sequence[np.ndarray], Vs: Sequence[np.ndarray],
                             scale: float, window: int, threads: int) -> List[np.ndarray]:
    """q [B, H_q, D]; Ks[b], Vs[b] [H_kv, L_b, D], all fp32.  Returns B arrays [H_q, D] (fp32)."""
    B = len(Ks)
    Hq = q.shape[1]
    outs = [np.zeros((Hq, q.shape[2]), dtype=np.float32) for _ in range(B)]

    def task(item):
        b, kv = item
        Hkv, L, _ = Ks[b].shape
        G = Hq // Hkv
        lo, hi = visible_range(L, window)
        if hi > lo:
            outs[b][kv * G:(kv + 1) * G] = _one_kv_head(q[b, kv * G:(kv + 1) * G], Ks[b][kv, lo:hi], Vs[b][kv, lo:hi], scale)

    items = [(b, kv) for b in range(B) for kv in range(Ks[b].shape[0])]
    with ThreadPoolExecutor(max_workers=max(1, threads)) as pool:
        list(pool.map(task, items))
    return outs
