"""Pins of the attention oracle: brute force, closed forms, special cases, a library routine.

The brute force below is written with explicit Python loops and math.exp over
an MHA-expanded cache, not with the oracle's vectorised steps, so an index,
sign or transposition mistake in either shows up as a disagreement.
"""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle.attn import decode_attention_batch, decode_attention_one, visible_range

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_examples.json")))


def brute_force(q, K, V, scale, window):
    Hq, D = len(q), len(q[0])
    Hkv, L = len(K), len(K[0])
    G = Hq // Hkv
    first = 0 if window <= 0 else max(0, L - window)
    out = [[0.0] * D for _ in range(Hq)]
    for h in range(Hq):
        kv = h // G
        scores = []
        for t in range(first, L):
            acc = 0.0
            for d in range(D):
                acc += q[h][d] * K[kv][t][d]
            scores.append(scale * acc)
        if not scores:
            continue
        big = max(scores)
        weights = [math.exp(s - big) for s in scores]
        tot = sum(weights)
        for d in range(D):
            acc = 0.0
            for j, t in enumerate(range(first, L)):
                acc += weights[j] * V[kv][t][d]
            out[h][d] = acc / tot
    return np.array(out)


def rand_case(rng, Hq, Hkv, L, D):
    return (rng.normal(size=(Hq, D)), rng.normal(size=(Hkv, L, D)), rng.normal(size=(Hkv, L, D)))


@pytest.mark.parametrize("Hq,Hkv,L,D,window", [
    (4, 2, 1, 8, 0), (4, 2, 7, 8, 0), (4, 2, 37, 16, 5), (6, 3, 20, 4, 20), (8, 2, 33, 8, 32),
    (4, 4, 19, 8, 3), (2, 1, 50, 8, 100)])
def test_against_brute_force(Hq, Hkv, L, D, window):
    rng = np.random.default_rng(Hq * 1000 + L)
    q, K, V = rand_case(rng, Hq, Hkv, L, D)
    scale = 1.0 / math.sqrt(D)
    got = decode_attention_one(q, K, V, scale, window)
    want = brute_force(q.tolist(), K.tolist(), V.tolist(), scale, window)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_window_timeline_example():
    g = GOLD["window_timeline"]
    toks = g["cached_after_append"]
    lo, hi = visible_range(len(toks), g["window"])
    assert toks[lo:hi] == g["read"]
    assert visible_range(5, 0) == (0, 5)
    assert visible_range(3, 8) == (0, 3)
    assert visible_range(0, 4) == (0, 0)


def test_single_token_returns_its_value():
    rng = np.random.default_rng(0)
    q, K, V = rand_case(rng, 4, 2, 1, 16)
    out = decode_attention_one(q, K, V, 0.3, 0)
    for h in range(4):
        assert np.array_equal(out[h], V[h // 2, 0])


def test_equal_keys_give_mean_of_visible_values():
    rng = np.random.default_rng(1)
    q, K, V = rand_case(rng, 4, 2, 24, 8)
    K[:] = K[:, :1, :]
    out = decode_attention_one(q, K, V, 0.7, 0)
    np.testing.assert_allclose(out[0], V[0].mean(axis=0), rtol=1e-13)
    outw = decode_attention_one(q, K, V, 0.7, 5)
    np.testing.assert_allclose(outw[3], V[1, -5:].mean(axis=0), rtol=1e-13)


def test_window_not_smaller_than_length_is_full_attention():
    rng = np.random.default_rng(2)
    q, K, V = rand_case(rng, 4, 2, 30, 8)
    full = decode_attention_one(q, K, V, 0.4, 0)
    assert np.array_equal(full, decode_attention_one(q, K, V, 0.4, 30))
    assert np.array_equal(full, decode_attention_one(q, K, V, 0.4, 31))
    assert not np.allclose(full, decode_attention_one(q, K, V, 0.4, 29))


def test_window_boundary_is_exact():
    """A token just outside the window must not contribute; the first one inside must."""
    rng = np.random.default_rng(3)
    Hq, Hkv, L, D, W = 2, 1, 40, 8, 16
    q, K, V = rand_case(rng, Hq, Hkv, L, D)
    base = decode_attention_one(q, K, V, 1.0, W)
    V2 = V.copy()
    V2[:, L - W - 1] += 1e6                         # just outside
    assert np.array_equal(base, decode_attention_one(q, K, V2, 1.0, W))
    V3 = V.copy()
    V3[:, L - W] += 1.0                             # first inside
    assert not np.allclose(base, decode_attention_one(q, K, V3, 1.0, W))
    K4, V4 = K.copy(), V.copy()
    K4[:, :L - W] = np.nan
    V4[:, :L - W] = np.nan                          # nothing outside is even read
    assert np.array_equal(base, decode_attention_one(q, K4, V4, 1.0, W))


def test_gqa_group_mapping():
    rng = np.random.default_rng(4)
    Hq, Hkv, L, D = 8, 2, 21, 8
    q, K, V = rand_case(rng, Hq, Hkv, L, D)
    q[1] = q[0]
    q[5] = q[4]
    out = decode_attention_one(q, K, V, 0.5, 0)
    assert np.array_equal(out[0], out[1]) and np.array_equal(out[4], out[5])
    # GQA equals MHA on a cache in which every KV head is repeated G times, in order
    G = Hq // Hkv
    Krep, Vrep = np.repeat(K, G, axis=0), np.repeat(V, G, axis=0)
    np.testing.assert_array_equal(out, decode_attention_one(q, Krep, Vrep, 0.5, 0))
    # and head h must use KV head h // G, not h % Hkv
    V2 = V.copy()
    V2[1] += 100.0
    out2 = decode_attention_one(q, K, V2, 0.5, 0)
    changed = [not np.allclose(out[h], out2[h]) for h in range(Hq)]
    assert changed == [False] * 4 + [True] * 4


def test_peaked_softmax_selects_argmax_token():
    rng = np.random.default_rng(5)
    Hq, Hkv, L, D = 2, 1, 17, 8
    q, K, V = rand_case(rng, Hq, Hkv, L, D)
    q[:] = 0.0
    q[:, 3] = 1.0
    out = decode_attention_one(q, K, V, 1e4, 0)
    t = int(np.argmax(K[0, :, 3]))
    np.testing.assert_allclose(out[0], V[0, t], rtol=1e-9, atol=1e-12)


def test_invariances_of_softmax_attention():
    rng = np.random.default_rng(6)
    Hq, Hkv, L, D = 4, 2, 26, 8
    q, K, V = rand_case(rng, Hq, Hkv, L, D)
    out = decode_attention_one(q, K, V, 0.9, 0)
    perm = rng.permutation(L)                        # order of the visible tokens is irrelevant
    np.testing.assert_allclose(out, decode_attention_one(q, K[:, perm], V[:, perm], 0.9, 0),
                               rtol=1e-12, atol=1e-14)
    c = rng.normal(size=D)                           # a common key offset shifts every score equally
    np.testing.assert_allclose(out, decode_attention_one(q, K + c, V, 0.9, 0), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(out + 2.5, decode_attention_one(q, K, V + 2.5, 0.9, 0), rtol=1e-12)
    np.testing.assert_allclose(3.0 * out, decode_attention_one(q, K, 3.0 * V, 0.9, 0), rtol=1e-12)
    # scale multiplies the logits: scale s on q equals scale 1 on s*q
    np.testing.assert_allclose(out, decode_attention_one(0.9 * q, K, V, 1.0, 0), rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("window", [0, 9, 64])
def test_against_library_sdpa(window):
    """Third opinion: torch's scaled_dot_product_attention on CPU with an explicit mask."""
    rng = np.random.default_rng(7)
    Hq, Hkv, L, D = 6, 3, 45, 16
    q, K, V = rand_case(rng, Hq, Hkv, L, D)
    scale = 1.0 / math.sqrt(D)
    got = decode_attention_one(q, K, V, scale, window)
    G = Hq // Hkv
    tq = torch.from_numpy(q)[None, :, None, :]                       # [1, Hq, 1, D]
    tk = torch.from_numpy(np.repeat(K, G, axis=0))[None]             # [1, Hq, L, D]
    tv = torch.from_numpy(np.repeat(V, G, axis=0))[None]
    mask = torch.zeros(1, 1, 1, L, dtype=torch.bool)
    lo = 0 if window <= 0 else max(0, L - window)
    mask[..., lo:] = True
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=scale)
    np.testing.assert_allclose(got, ref[0, :, 0, :].numpy(), rtol=1e-10, atol=1e-12)


def test_batch_wrapper_and_empty():
    rng = np.random.default_rng(8)
    q = rng.normal(size=(3, 4, 8))
    Ks = [rng.normal(size=(2, L, 8)) for L in (5, 1, 12)]
    Vs = [rng.normal(size=(2, L, 8)) for L in (5, 1, 12)]
    out = decode_attention_batch(q, Ks, Vs, 0.5, 4)
    for b in range(3):
        assert np.array_equal(out[b], decode_attention_one(q[b], Ks[b], Vs[b], 0.5, 4))
    empty = decode_attention_one(q[0], np.zeros((2, 0, 8)), np.zeros((2, 0, 8)), 0.5, 0)
    assert np.array_equal(empty, np.zeros((4, 8)))


def test_threaded_fp32_baseline_agrees_with_the_oracle():
    """The second CPU baseline of the benchmark's report computes what the oracle computes."""
    from oracle.attn_threads import decode_attention_threads
    rng = np.random.default_rng(11)
    for window in (0, 37):
        lens = [1, 5, 64, 300, 1000]
        q = rng.normal(size=(len(lens), 8, 64)).astype(np.float32)
        Ks = [rng.normal(size=(2, L, 64)).astype(np.float32) for L in lens]
        Vs = [rng.normal(size=(2, L, 64)).astype(np.float32) for L in lens]
        got = decode_attention_threads(q, Ks, Vs, 0.125, window, threads=3)
        for b in range(len(lens)):
            want = decode_attention_one(q[b], Ks[b], Vs[b], 0.125, window)
            assert np.abs(got[b] - want).max() <= 2e-6
