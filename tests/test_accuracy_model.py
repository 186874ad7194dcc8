"""What the regression bound of the GPU parity tests can and cannot see (CPU only).

A numpy model of the ARITHMETIC of the bf16 decode path -- not of its code: bf16 inputs multiplied
exactly and accumulated in fp32, scores in the base-2 domain, exp2 of (score - maximum) in fp32,
the normaliser summed from the unrounded weights, and the weights entering the value product
rounded to bf16 -- run once with the weight as the sum of two bf16 numbers (its rounding and
the rounding of the remainder: what the kernels do) and once with the first term only.  Against
the fp64 oracle on the same inputs the two-term form stays far inside the regression bound of
tests/test_gpu_parity.py and the one-term form breaks it, while both pass the stated tolerance
of 2e-2: the regression bound is what notices the difference.
"""
import math

import numpy as np
import torch

from oracle.attn import decode_attention_one

from test_gpu_parity import REG_BF16_ABS, TOL_BF16_ABS


def bf16_round(x: np.ndarray) -> np.ndarray:
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).bfloat16().float().numpy()


def model_bf16_path(q, K, V, scale, two_term: bool) -> np.ndarray:
    """q [H, D], K, V [L, D] (one KV head, already bf16-representable), fp32 arithmetic."""
    q, K, V = (np.asarray(x, dtype=np.float32) for x in (q, K, V))
    s2 = (K @ q.T).T * np.float32(scale * math.log2(math.e))            # [H, L] fp32
    m = s2.max(axis=1, keepdims=True)
    e = np.exp2(s2 - m).astype(np.float32)
    l = e.sum(axis=1, dtype=np.float32)
    hi = bf16_round(e)
    acc = hi @ V
    if two_term:
        acc = acc + bf16_round(e - hi) @ V
    return (acc / l[:, None]).astype(np.float64)


def test_one_term_probabilities_break_the_regression_bound_two_terms_do_not():
    rng = np.random.default_rng(5)
    D, H = 128, 4
    worst = {True: 0.0, False: 0.0}
    for L in [2, 3, 5, 9, 16, 17, 40, 100, 333, 700] * 3:
        q = bf16_round(rng.normal(size=(H, D)))
        K = bf16_round(rng.normal(size=(L, D)))
        V = bf16_round(rng.normal(size=(L, D)))
        want = decode_attention_one(q, K[None], V[None], 1 / math.sqrt(D), 0)
        for two in (True, False):
            err = float(np.abs(model_bf16_path(q, K, V, 1 / math.sqrt(D), two) - want).max())
            worst[two] = max(worst[two], err)
    assert worst[True] <= REG_BF16_ABS / 10          # two terms: a few 1e-6
    assert worst[False] > 10 * REG_BF16_ABS          # one term: about 2^-9 of |V|
    assert worst[False] <= TOL_BF16_ABS              # ... which the stated tolerance alone lets through
