"""Pins of the allocator oracle against what the paper prints and what its text mandates.

None of these re-types the oracle's own code path: they are worked examples of
the paper (tests/golden/paper_examples.json), closed forms, and invariants
checked from the outside (byte extents, ownership) after every operation.
"""
import json
import os

import numpy as np
import pytest

from oracle.alloc import (InvalidOp, OraclePool, OracleRequests, OutOfPages,
                          first_needed_token, kv_small_page_bytes, lcm_bytes)
from workloads import configs, scripts

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_examples.json")))


# ---------------------------------------------------------------- LCM / split
def test_lcm_intro_example():
    g = GOLD["lcm_intro"]
    assert lcm_bytes(g["sizes"]) == g["large"]


def test_lcm_mllama_figure_sizes_and_split():
    g = GOLD["lcm_mllama_figure"]
    # footnote: per-token KV of one layer is 128; tokens_per_page = 1
    img = g["per_layer_kv"] * g["cross_layers"]
    txt = g["per_layer_kv"] * g["self_layers"]
    assert (img, txt) == (g["image_page"], g["text_page"])
    pool = OraclePool(10 * g["large"], [img, txt])
    assert pool.large_bytes == g["large"]
    assert pool.r == [3, 2]
    assert all(rk * s == pool.large_bytes for rk, s in zip(pool.r, pool.S))


def test_small_page_bytes_formula_matches_footnote_and_kv_size_example():
    # footnote shape: "KV size per token of each layer is 128" -> e.g. 1 kv head, D=32, 2 B, K+V
    assert kv_small_page_bytes(2, 1, 32, 1, 2) == 256
    assert kv_small_page_bytes(3, 1, 32, 1, 2) == 384
    # Sec. 2: Llama 3.1 8B (32 layers, 8 KV heads, head_dim 128, 16-bit) at 10k tokens ~ 1.2 GB
    g = GOLD["kv_size_llama31_8b"]
    total = kv_small_page_bytes(32, 8, 128, 1, 2) * g["tokens"]
    assert abs(total / 2 ** 30 - g["approx_GB"]) < 0.05


@pytest.mark.parametrize("name", list(configs.ALL))
def test_large_page_splits_exactly_for_every_config(name):
    cfg = configs.ALL[name]()
    S = [k.small_page_bytes for k in cfg.kinds]
    L = lcm_bytes(S)
    pool = OraclePool(4 * L, S)
    for k, s in enumerate(S):
        assert pool.r[k] * s == L and L % s == 0
    # L is the *least* common multiple: no proper divisor of it is a common multiple
    for d in range(2, 64):
        if L % d == 0:
            assert any((L // d) % s for s in S)


def test_expected_geometry_of_the_five_configs():
    KiB = 1024
    want = {
        "tiny": ([16 * KiB, 32 * KiB], 32 * KiB, [2, 1]),
        "gemma2_9b": ([2688 * KiB, 2688 * KiB], 2688 * KiB, [1, 1]),
        "llama32_vision_11b": ([2048 * KiB, 512 * KiB], 2048 * KiB, [1, 4]),
        "jamba_like": ([256 * KiB, 14336 * KiB], 14336 * KiB, [56, 1]),
        "long_5to1": ([2560 * KiB, 512 * KiB], 2560 * KiB, [1, 5]),
    }
    for name, (S, L, r) in want.items():
        cfg = configs.ALL[name]()
        assert [k.small_page_bytes for k in cfg.kinds] == S
        pool = OraclePool(2 * L, S)
        assert pool.large_bytes == L and pool.r == r
    lit = configs.jamba_like(literal=True)
    assert [k.small_page_bytes for k in lit.kinds] == [64 * KiB, 512 * KiB]
    assert OraclePool(2 ** 20, [k.small_page_bytes for k in lit.kinds]).r == [8, 1]


# ------------------------------------------------- Fig. two_level_overview
def test_two_level_overview_figure():
    g = GOLD["two_level_overview"]
    IMG, TXT, R = 0, 1, 7
    pool = OraclePool(8 * 768, [256, 384])
    order = [IMG, TXT, IMG, IMG, TXT, IMG]          # the call order is ours; the sets are the paper's
    ids = {IMG: [], TXT: []}
    for k in order:
        ids[k].append(pool.alloc(k, R))
    assert len(ids[IMG]) == g["image_small_pages"] and len(ids[TXT]) == g["text_small_pages"]
    assert sorted({i // pool.r[IMG] for i in ids[IMG]}) == g["image_large_pages"]
    assert sorted({i // pool.r[TXT] for i in ids[TXT]}) == g["text_large_pages"]
    assert sorted(ids[TXT]) == g["text_small_ids"]
    # ids are byte offsets in units of the type's own page size (Sec. 4.1 / 4.2)
    for t in ids[TXT]:
        assert 768 <= pool.byte_offset(TXT, t) < 2 * 768
    assert ids[IMG] == [0, 1, 2, 6]


# ------------------------------------------------- allocate()/free() contract
def test_split_on_demand_and_return_when_all_unused():
    pool = OraclePool(3 * 768, [256, 384])
    assert pool.free_large() == 3
    a = pool.alloc(0, 1)
    assert pool.free_large() == 2 and pool.owned_large(0) == 1
    b = pool.alloc(0, 1)
    c = pool.alloc(0, 1)
    assert pool.free_large() == 2                     # still the same large page
    d = pool.alloc(0, 1)
    assert pool.free_large() == 1                     # fourth one needs a second large page
    pool.free(0, a); pool.free(0, b)
    assert pool.free_large() == 1                     # c still lives there
    pool.free(0, c)
    assert pool.free_large() == 2                     # returned at once
    pool.free(0, d)
    assert pool.free_large() == 3 and pool.owned_large(0) == 0


def test_returned_large_page_can_change_type():
    pool = OraclePool(1 * 768, [256, 384])
    a = pool.alloc(0, 1)
    with pytest.raises(OutOfPages):
        pool.alloc(1, 1)                              # the only large page belongs to kind 0
    pool.free(0, a)
    t = pool.alloc(1, 1)                              # same bytes, now text pages
    assert t == 0 and pool.large_owner(0) == (1, 1)


def test_errors():
    pool = OraclePool(2 * 768, [256, 384])
    a = pool.alloc(0, 1)
    pool.free(0, a)
    with pytest.raises(InvalidOp):
        pool.free(0, a)
    with pytest.raises(InvalidOp):
        pool.ref(0, a)
    with pytest.raises(InvalidOp):
        pool.alloc(2, 1)
    with pytest.raises(InvalidOp):
        pool.free(0, 10 ** 6)
    with pytest.raises(InvalidOp):
        OraclePool(768, [256, 384], large_page_bytes=1000)


def test_refcount_keeps_page_alive():
    pool = OraclePool(2 * 768, [256, 384])
    a = pool.alloc(1, 1)
    pool.ref(1, a)
    pool.free(1, a)
    assert pool.used_small(1) == 1 and pool.free_large() == 1
    pool.free(1, a)
    assert pool.used_small(1) == 0 and pool.free_large() == 2


# ------------------------------------------------- Sec. 4.3 three-step order
def test_step1_prefers_own_large_page():
    pool = OraclePool(4 * 1024, [256, 1024])          # kind 0: r = 4
    a0 = pool.alloc(0, 1)                             # large 0 -> request 1
    b0 = pool.alloc(0, 2)                             # step 1 fails for request 2, step 2: large 1
    a1 = pool.alloc(0, 1)
    b1 = pool.alloc(0, 2)
    assert [a0, a1] == [0, 1] and [b0, b1] == [4, 5]
    assert pool.large_owner(0) == (0, 1) and pool.large_owner(1) == (0, 2)


def test_step2_before_step3_and_step3_when_no_large_page_left():
    pool = OraclePool(2 * 1024, [256, 1024])          # two large pages, kind 0: r = 4
    a = pool.alloc(0, 1)                              # large 0 (3 unused slots remain)
    b = pool.alloc(0, 2)                              # step 2 preferred over stealing: large 1
    assert b == 4
    c = pool.alloc(0, 3)                              # no large page left: step 3, lowest page, lowest slot
    assert c == 1
    assert pool.large_owner(0) == (0, 1)              # association unchanged by the theft
    # fill everything, then OOM
    for _ in range(5):
        pool.alloc(0, 3)
    with pytest.raises(OutOfPages):
        pool.alloc(0, 3)
    # the association outlives its owner's pages while a stolen slot is live
    pool.free(0, a)
    assert pool.large_owner(0) == (0, 1)


def test_internal_frag_figure_request_aware_vs_naive():
    g = GOLD["internal_frag"]
    r = g["small_per_large"]
    n_each = 8

    def run(policy):
        pool = OraclePool(16 * r * 64, [64, r * 64], policy=policy)
        assert pool.r == [r, 1]
        mine = {1: [], 2: []}
        for _ in range(n_each):                       # A and B allocate interleaved
            for req in (1, 2):
                mine[req].append(pool.alloc(0, req))
        before = pool.free_large()
        for sid in mine[1]:                           # A completes: its pages go together
            pool.free(0, sid)
        return pool.free_large() - before

    assert run("request_aware") == n_each // r        # every large page of A comes back
    assert run("naive") == 0                          # every large page still holds pages of B


def test_no_mixing_without_step3():
    """With large pages to spare, a large page only ever holds one request's pages."""
    ops = scripts.lowlevel_trace(n_kinds=2, n_requests=6, n_ops=600, seed=5, p_ref=0.0)
    pool = OraclePool(4096 * 768, [256, 384])
    h2 = {}
    owner = {}
    for op in ops:
        if op[0] == "alloc":
            _, h, k, req = op
            sid = pool.alloc(k, req)
            h2[h] = (k, sid)
            owner[(k, sid)] = req
            large = sid // pool.r[k]
            assert pool.large_owner(large) == (k, req)
        elif op[0] == "unref":
            k, sid = h2[op[1]]
            pool.free(k, sid)
            del owner[(k, sid)]
    assert pool.free_large() == pool.n_large


# ------------------------------------------------- invariants on random traces
def _check_invariants(pool):
    ext = sorted(pool.live_extents())
    for (b0, e0, _, _), (b1, e1, _, _) in zip(ext, ext[1:]):
        assert e0 <= b1, "two live small pages overlap in bytes"
    kinds_in_large = {}
    for b, e, k, sid in ext:
        large = b // pool.large_bytes
        assert (e - 1) // pool.large_bytes == large, "small page straddles large pages"
        assert e <= pool.n_large * pool.large_bytes
        kinds_in_large.setdefault(large, set()).add(k)
        assert pool.large_owner(large)[0] == k
    assert all(len(s) == 1 for s in kinds_in_large.values())
    owned = sum(pool.owned_large(k) for k in range(len(pool.S)))
    assert owned + pool.free_large() == pool.n_large
    assert owned == len(kinds_in_large), "a large page is held with no live small page"


@pytest.mark.parametrize("seed,sizes,n_large", [
    (1, [256, 384], 12), (2, [16384, 32768], 16), (3, [2048, 3072, 6144], 10),
    (4, [512 * 1024, 2048 * 1024], 6), (5, [4096, 28672 * 8], 5)])
def test_invariants_after_every_op(seed, sizes, n_large):
    L = lcm_bytes(sizes)
    pool = OraclePool(n_large * L + 17, sizes)        # a ragged tail of bytes is never used
    assert pool.n_large == n_large
    ops = scripts.lowlevel_trace(len(sizes), 5, 400, seed)
    h2 = {}
    refs = {}
    ooms = 0
    for op in ops:
        if op[0] == "alloc":
            _, h, k, req = op
            try:
                h2[h] = (k, pool.alloc(k, req))
                refs[h] = 1
            except OutOfPages:
                ooms += 1
                refs[h] = 0
        elif op[0] == "ref":
            if refs.get(op[1], 0) > 0:
                pool.ref(*h2[op[1]])
                refs[op[1]] += 1
        elif op[0] == "unref":
            if refs.get(op[1], 0) > 0:
                pool.free(*h2[op[1]])
                refs[op[1]] -= 1
        _check_invariants(pool)
    assert pool.free_large() == pool.n_large and pool.used_bytes() == 0   # freeing all empties the pool
    assert all((rc == 0).all() for rc in pool.refcount)


# ------------------------------------------------- accounting closed forms (Sec. 3.2)
def test_mllama_waste_closed_form():
    g = GOLD["mllama_waste"]
    E = 128
    T_txt, I_img = g["text_tokens"], g["image_tokens"]
    S_self = E * g["self_layers"]                     # tokens_per_page = 1, as in the paper's figures
    S_cross = E * g["cross_layers"]
    pool = OraclePool(2200 * 4096, [S_self, S_cross])
    reqs = OracleRequests(pool, [1, 1], [0, 0])
    reqs.extend(1, 0, T_txt)
    reqs.extend(1, 1, I_img)
    ideal = pool.used_bytes()
    assert ideal == (T_txt * g["self_layers"] + I_img * g["cross_layers"]) * E
    homogeneous = (T_txt + I_img) * (g["self_layers"] + g["cross_layers"]) * E
    waste = 100.0 * (1 - ideal / homogeneous)
    assert round(waste, 1) == g["waste_percent"]


@pytest.mark.parametrize("n_full,n_win,W,L,key", [
    (21, 21, 4096, 8192, "gemma2_percent"),           # Gemma-2: alternate layers, 8k context
    (9, 27, 32768, 131072, "ministral_percent"),      # Ministral: 3 of 4 layers windowed, 128k
])
def test_window_waste_closed_form(n_full, n_win, W, L, key):
    E, T = 64, 16
    S = [E * n_full * T, E * n_win * T]
    pool = OraclePool((2 * L // T + 64) * lcm_bytes(S), S)   # extend allocates, then slides out
    reqs = OracleRequests(pool, [T, T], [0, W])
    reqs.extend(1, 0, L)
    reqs.extend(1, 1, L)
    ideal = pool.used_bytes()
    homogeneous = L * (n_full + n_win) * E
    assert 100.0 * (1 - ideal / homogeneous) == GOLD["window_waste"][key]


# ------------------------------------------------- window need set and slide-out
def test_window_timeline_example():
    g = GOLD["window_timeline"]
    toks = g["cached_after_append"]
    lo = first_needed_token(len(toks), g["window"])
    assert toks[lo:] == g["read"]
    assert first_needed_token(3, 0) == 0 and first_needed_token(1, 2) == 0


@pytest.mark.parametrize("W,T", [(32, 16), (40, 16), (2, 1), (100, 8)])
def test_resident_window_pages_are_exactly_those_touching_the_window(W, T):
    pool = OraclePool(64 * 1024, [1024])
    reqs = OracleRequests(pool, [T], [W])
    rng = np.random.default_rng(W * 131 + T)
    L = 0
    while L < 700:
        L += int(rng.integers(1, 3 * T))
        reqs.extend(9, 0, L)
        row = reqs.pages[(9, 0)]
        lo = max(0, L - W)
        for p, sid in enumerate(row):
            touches = p * T < L and (p + 1) * T > lo
            assert (sid >= 0) == touches
    reqs.free_request(9)
    assert pool.free_large() == pool.n_large


@pytest.mark.parametrize("T", [1, 16, 24])
def test_a_partly_filled_last_page_is_a_page(T):
    """Every cached token lies in a page (Sec. 4.2: a token is addressed by page id and offset in
    the page): L tokens take ceil(L / T) pages, not floor, and growing inside a page takes none."""
    pool = OraclePool(64 * 512, [512])
    reqs = OracleRequests(pool, [T], [0])
    want = 0
    for L in (1, T, T + 1, 2 * T, 3 * T - 1 if T > 1 else 5, 3 * T + 1):
        reqs.extend(7, 0, L)
        want = max(want, (L + T - 1) // T)
        assert pool.used_small(0) == want == len(reqs.row(7, 0, want))
        assert all(x >= 0 for x in reqs.row(7, 0, want))


def test_a_table_row_marks_what_is_not_resident():
    """The block-table row of a request (Sec. 4.2, the per-type page list): its pages in logical
    order, then -1 for every column past them, and -1 where a window page slid out -- never an id,
    which would name a page that belongs to someone else."""
    pool = OraclePool(16 * 512, [512])
    reqs = OracleRequests(pool, [4], [6])             # 4 tokens per page, window of 6 tokens
    reqs.extend(1, 0, 4)                              # another request holds page 0
    reqs.extend(2, 0, 9)                              # pages 1, 2, 3
    assert reqs.row(2, 0, 6) == [1, 2, 3, -1, -1, -1]
    reqs.extend(2, 0, 14)                             # tokens 8..13 are needed: logical pages 0 and 1 slid out
    assert reqs.row(2, 0, 6) == [-1, -1, 3, 4, -1, -1]
    with pytest.raises(InvalidOp):
        reqs.row(2, 0, 3)


def test_share_prefix_and_free_order():
    pool = OraclePool(64 * 4096, [1024, 4096])
    reqs = OracleRequests(pool, [16, 16], [0, 0])
    reqs.extend(1, 0, 100)
    reqs.share_prefix(1, 2, 0, 4)
    assert reqs.pages[(2, 0)] == reqs.pages[(1, 0)][:4]
    reqs.extend(2, 0, 130)
    assert len(set(reqs.pages[(2, 0)][4:]) & set(reqs.pages[(1, 0)])) == 0
    reqs.free_request(1)
    assert all(pool.refcount[0][s] == 1 for s in reqs.pages[(2, 0)])
    reqs.free_request(2)
    assert pool.free_large() == pool.n_large


# ------------------------------------------------- the workload scripts fit and drain
def test_tiny_script_fits_the_64_page_pool_and_drains():
    cfg = configs.tiny()
    for seed in range(5):
        ctx = scripts.sample_ctx(cfg, seed)
        S = [k.small_page_bytes for k in cfg.kinds]
        pool = OraclePool(cfg.pool_large_pages * lcm_bytes(S), S)
        reqs = OracleRequests(pool, [k.tokens_per_page for k in cfg.kinds],
                              [k.window for k in cfg.kinds])
        scripts.run_script(scripts.build_script(cfg, ctx, seed), reqs)
        scripts.run_script(scripts.step_script(cfg, ctx), reqs)
        # window kind: at most 3 resident pages per request (window 32, page 16)
        for b in range(cfg.batch):
            row = reqs.pages[(scripts.request_id(b), 1)]
            assert sum(s >= 0 for s in row) <= 3
        scripts.run_script(scripts.finish_script(cfg, seed), reqs)
        assert pool.free_large() == pool.n_large
