"""Attention oracle: single-token decode attention over contiguous K/V, fp64.

TEST INFRASTRUCTURE ONLY (see the package docstring).

Paging is an addressing scheme, not an approximation (Sec. 4.2: the kernel is
handed start pointer, page size and page ids and computes attention "as
usual"), so what the paged path must reach is the plain definition, written
out here on unpaged tensors:

    out[h, :] = sum_{t in Vis} softmax_t( scale * <q[h, :], K[h // G, t, :]> ) * V[h // G, t, :]

with G = n_q_heads / n_kv_heads (grouped-query attention, Sec. 3.1 c) and the
visible set Vis
  * full attention:   [0, L)                 (Sec. 1, full-prefix dependency)
  * sliding window W: [max(0, L - W), L)     (Sec. 3.1 a, Sec. 5.1; Fig. last-access a:
                                             window 2 reads D, E to produce F)
  * cross attention:  [0, Lx), Lx the fixed number of encoder (image) tokens
                                             (Sec. 3.1 c)
L counts the tokens cached after this step's append, so the token being
decoded is the last visible one.

Everything is computed in float64 whatever the storage type of the inputs,
with a two-pass softmax (max, then exponentials, then one division).
"""
from __future__ import annotations

from typing import Tuple

import numpy as np


def visible_range(seq_len: int, window: int) -> Tuple[int, int]:
    """[lo, hi) of the token positions a query at length seq_len attends to."""
    if seq_len <= 0:
        return 0, 0
    if window and window > 0:
        return max(0, seq_len - window), seq_len
    return 0, seq_len


def decode_attention_one(q: np.ndarray, K: np.ndarray, V: np.ndarray,
                         scale: float, window: int = 0) -> np.ndarray:
    """One request, one layer.

    q [H_q, D]; K, V [H_kv, L, D] holding the L cached tokens in order (the
    newly appended one last).  Returns out [H_q, D] in float64.  An empty
    visible set gives zeros.
    """
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    Hq, D = q.shape
    Hkv, L, Dk = K.shape
    assert Dk == D and V.shape == K.shape and Hq % Hkv == 0
    G = Hq // Hkv
    lo, hi = visible_range(L, window)
    out = np.zeros((Hq, D), dtype=np.float64)
    if hi <= lo:
        return out
    for h in range(Hq):
        kv = h // G
        s = scale * (K[kv, lo:hi, :] @ q[h, :])        # [n_vis]
        m = s.max()
        e = np.exp(s - m)
        out[h, :] = (e @ V[kv, lo:hi, :]) / e.sum()
    return out


def decode_attention_batch(q, Ks, Vs, scale: float, window: int = 0) -> np.ndarray:
    """q [B, H_q, D]; Ks[b], Vs[b] are [H_kv, L_b, D].  Returns [B, H_q, D] fp64."""
    return np.stack([decode_attention_one(q[b], Ks[b], Vs[b], scale, window)
                     for b in range(len(Ks))])
