"""Pins of the oracle's prefix-cache side: page states, LRU keys, five-step allocation, hit rules.

Worked examples are the paper's (tests/golden/paper_examples.json); the rest are invariants and
the reduction to the three-step allocator when nothing is cached.
"""
import json
import os

import numpy as np
import pytest

from oracle.alloc import (EMPTY, EVICTABLE, USED, InvalidOp, OracleCachingPool, OraclePool, OutOfPages,
                          lcm_bytes, longest_common_prefix, possible_prefixes_every,
                          possible_prefixes_full, possible_prefixes_window)
from workloads import scripts

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_examples.json")))
FULL, WIN = 0, 1


def run_last_access_example(pool):
    """Sec. 5.1: two requests on one self-attention and one sliding-window (2) layer, one token per page."""
    g = GOLD["last_access_example"]
    tok = {}

    def touch(k, letters, t):
        for ch in letters:
            pool.set_last_access(k, tok[(k, ch)], t)

    # step 1: request 1 prefills ABCD
    for k in (FULL, WIN):
        for ch in g["request1"]["input"]:
            tok[(k, ch)] = pool.alloc(k, 1)
    touch(FULL, g["timeline"][0]["self"], 1)
    touch(WIN, g["timeline"][0]["window"], 1)
    # step 2: request 1 decodes: E's KV joins the cache (the generated F has none)
    for k in (FULL, WIN):
        tok[(k, "E")] = pool.alloc(k, 1)
    touch(FULL, g["timeline"][1]["self"], 2)
    touch(WIN, g["timeline"][1]["window"], 2)
    for k in (FULL, WIN):                        # request 1 completes; its pages stay cached
        for i, ch in enumerate("ABCDE"):
            pool.set_prefix_length(k, tok[(k, ch)], i + 1)
        for ch in "ABCDE":
            pool.release(k, tok[(k, ch)], keep_cached=True)
    # step 3: request 2 = ABCD G hits the cached prefix ABCD and adds G
    for k in (FULL, WIN):
        for ch in "ABCD":
            pool.acquire(k, tok[(k, ch)])
        tok[(k, "G")] = pool.alloc(k, 2)
    touch(FULL, g["timeline"][2]["self"], 3)
    touch(WIN, g["timeline"][2]["window"], 3)
    for k in (FULL, WIN):
        for ch, n in zip("ABCDG", g["stated"]["prefix_lengths_ABCDG"]):
            pool.set_prefix_length(k, tok[(k, ch)], n)
        for ch in "ABCDG":
            pool.release(k, tok[(k, ch)], keep_cached=True)
    return tok


def test_last_access_times_of_the_paper_example():
    g = GOLD["last_access_example"]
    pool = OracleCachingPool(16 * 64, [64, 64])
    tok = run_last_access_example(pool)
    ts = lambda k, ch: int(pool.last_access[k][tok[(k, ch)]])
    assert ts(FULL, "E") == ts(WIN, "E") == g["stated"]["E_timestamp"]
    for ch in "CDG":
        assert ts(FULL, ch) == ts(WIN, ch) == g["stated"]["CDG_timestamp"]
    # tokens outside the window keep an earlier time in the window layer only
    assert [ts(WIN, "A"), ts(WIN, "B")] == [1, 1] and [ts(FULL, "A"), ts(FULL, "B")] == [3, 3]
    assert all(pool.state(k, s) == EVICTABLE for (k, _), s in tok.items())


def test_eviction_order_of_the_paper_example():
    g = GOLD["last_access_example"]
    pool = OracleCachingPool(12 * 64, [64, 64])       # 12 pages: the 12 cached tokens fill the pool
    tok = run_last_access_example(pool)
    name = {(k, s): ("self" if k == FULL else "win", ch) for (k, ch), s in tok.items()}
    assert pool.free_large() == 0
    order = []
    for _ in range(12):
        _, ev = pool.alloc_evict(FULL, 99)
        assert len(ev) == 1
        order.append(name[ev[0]])
    pos = {x: i for i, x in enumerate(order)}
    for layer in ("self", "win"):
        for later in g["stated"]["E_evicted_before"]:          # E (time 2) before C, D, G (time 3)
            assert pos[(layer, "E")] < pos[(layer, later)]
        for later in g["stated"]["G_evicted_before"]:          # equal times: longest prefix first
            assert pos[(layer, "G")] < pos[(layer, later)]
    # the window layer gives up the tokens outside its window before anything else
    assert set(order[:2]) == {("win", "A"), ("win", "B")} and order[0] == ("win", "B")
    with pytest.raises(OutOfPages):
        pool.alloc_evict(FULL, 99)


def test_each_of_the_five_steps_in_order():
    assert len(GOLD["five_steps"]["order"]) == 5
    pool = OracleCachingPool(3 * 1024, [256, 1024])   # kind 0: 4 small pages per large page
    a = [pool.alloc_evict(0, 1)[0] for _ in range(2)]             # step 2 then step 1
    assert a == [0, 1]
    b = pool.alloc_evict(0, 2)[0]                                  # step 2 (own large page) beats step 4
    assert b == 4
    c = pool.alloc_evict(1, 3)[0]                                  # last empty large page
    assert c == 2 and pool.free_large() == 0
    # large page 0 becomes {evictable, evictable, empty, empty}: by the definition of Sec. 5.4
    # ("evictable if all its small pages are evictable") it is NOT an evictable large page
    for t, sid in enumerate(a):
        pool.set_last_access(0, sid, 10 + t)
        pool.release(0, sid, keep_cached=True)
    # step 1 still wins for request 2 (its own large page has empty slots)
    assert pool.alloc_evict(0, 2) == (5, [])
    # request 7 has no page of its own and no empty large page exists; step 3 finds no evictable
    # large page (page 0 is mixed), so step 4 hands out an empty slot of another request's page
    # and nothing is evicted
    assert pool.alloc_evict(0, 7) == (2, [])
    assert pool.large_owner(0) == (0, 1)                           # the association stays request 1's
    assert [pool.state(0, s) for s in range(4)] == [EVICTABLE, EVICTABLE, USED, EMPTY]
    # kind 1 for request 8: steps 1-3 fail (no evictable large page), 4 and 5 find nothing of kind 1
    with pytest.raises(OutOfPages):
        pool.alloc_evict(1, 8)
    # step 4 again fills the page; released with their contents kept, all four small pages of
    # large page 0 are evictable and so is the large page
    assert pool.alloc_evict(0, 7) == (3, [])
    for sid, t in ((2, 3), (3, 4)):
        pool.set_last_access(0, sid, t)
        pool.release(0, sid, keep_cached=True)
    # step 3: kind 1 evicts large page 0 (all of its small pages are reported) and re-types it
    sid, ev = pool.alloc_evict(1, 8)
    assert sid == 0 and sorted(ev) == [(0, 0), (0, 1), (0, 2), (0, 3)] and pool.large_owner(0) == (1, 8)
    assert [pool.state(0, s) for s in range(4)] == [EMPTY] * 4
    # kind 0 owns large page 1 only: {used, used, empty, empty}; step 4 fills it for request 9
    assert [pool.alloc_evict(0, 9) for _ in range(2)] == [(6, []), (7, [])]
    pool.set_last_access(0, 6, 5)
    pool.release(0, 6, keep_cached=True)              # large page 1 still has used pages
    assert pool.alloc_evict(0, 10) == (6, [(0, 6)])   # steps 1-4 fail, step 5 evicts the small page
    with pytest.raises(OutOfPages):
        pool.alloc_evict(0, 10)


def test_large_page_is_evictable_only_when_all_its_small_pages_are():
    """Sec. 5.4: a large page is evictable if all its small pages are evictable.  One empty or one
    used small page keeps it out of step 3, for its own kind and for any other."""
    for spoiler in ("empty", "used"):
        pool = OracleCachingPool(2 * 1024, [256, 1024])
        x = [pool.alloc(0, 1) for _ in range(4)]      # large page 0, kind 0
        assert pool.alloc(1, 2) == 1                  # large page 1, kind 1
        for sid in x[:3]:
            pool.set_last_access(0, sid, 1)
            pool.release(0, sid, keep_cached=True)
        if spoiler == "empty":
            pool.release(0, x[3], keep_cached=False)
        with pytest.raises(OutOfPages):               # kind 1 cannot get large page 0
            pool.alloc_evict(1, 3)
        if spoiler == "empty":
            assert pool.alloc_evict(0, 3) == (x[3], [])              # step 4 (empty slot), no eviction
        else:
            assert pool.alloc_evict(0, 3) == (x[0], [(0, x[0])])     # step 5: one small page, lowest id among equal keys
        assert pool.large_owner(0) == (0, 1)
    # with the fourth page evictable too the large page goes as a whole, its LRU time being the
    # latest last access among ALL its small pages
    pool = OracleCachingPool(3 * 1024, [256, 1024])
    x = [pool.alloc(0, 1) for _ in range(4)]
    y = [pool.alloc(0, 2) for _ in range(4)]
    assert pool.alloc(1, 3) == 2
    for sid, t in zip(x, (1, 1, 1, 8)):
        pool.set_last_access(0, sid, t)
    for sid, t in zip(y, (7, 7, 7, 7)):
        pool.set_last_access(0, sid, t)
    for sid in x + y:
        pool.release(0, sid, keep_cached=True)
    sid, ev = pool.alloc_evict(1, 4)
    assert sid == 1 and sorted(ev) == [(0, s) for s in y]


def evictable_large_page_beats_another_requests_empty_slot(pool):
    """Sec. 5.4 orders the steps: an evictable large page is evicted (step 3) before an empty small
    page associated with another request is taken (step 4)."""
    x = [pool.alloc(0, 1) for _ in range(4)]          # large page 0, request 1
    y = pool.alloc(0, 2)                              # large page 1, request 2: three empty slots left
    z = pool.alloc(1, 3)                              # large page 2, the other kind: no empty large page left
    for sid in x:
        pool.set_last_access(0, sid, 4)
        pool.release(0, sid, keep_cached=True)        # large page 0: all four evictable
    got = pool.alloc_evict(0, 9)                      # request 9 owns nothing: steps 1 and 2 fail
    return x, y, z, got


def test_step_3_comes_before_step_4():
    x, y, z, got = evictable_large_page_beats_another_requests_empty_slot(OracleCachingPool(3 * 1024, [256, 1024]))
    assert (x, y, z) == ([0, 1, 2, 3], 4, 2)
    sid, ev = got
    assert sid == 0 and sorted(ev) == [(0, 0), (0, 1), (0, 2), (0, 3)]      # not slot 5 of request 2's page


def small_pages_of_equal_age(pool):
    """Sec. 5.1: among tokens of equal last access the one with the highest prefix length goes
    first -- also when single small pages are evicted (step 5)."""
    x = [pool.alloc(0, 1) for _ in range(4)]          # one large page; page x[0] stays in use
    for sid, n in zip(x[1:], (2, 7, 4)):
        pool.set_last_access(0, sid, 5)
        pool.set_prefix_length(0, sid, n)
        pool.release(0, sid, keep_cached=True)
    return x, [pool.alloc_evict(0, 9) for _ in range(3)]


def test_step_5_ties_go_to_the_longest_prefix():
    x, got = small_pages_of_equal_age(OracleCachingPool(1024, [256], 1024))
    assert x == [0, 1, 2, 3]
    assert got == [(2, [(0, 2)]), (3, [(0, 3)]), (1, [(0, 1)])]            # prefix 7, then 4, then 2


def test_large_page_lru_uses_latest_access_of_its_small_pages():
    pool = OracleCachingPool(2 * 1024, [256, 1024])
    x = [pool.alloc(0, 1) for _ in range(4)]          # large page 0
    y = [pool.alloc(0, 2) for _ in range(4)]          # large page 1
    for sid, t in zip(x, (1, 1, 1, 9)):               # one recently used page keeps page 0 young
        pool.set_last_access(0, sid, t)
    for sid, t in zip(y, (5, 5, 5, 5)):
        pool.set_last_access(0, sid, t)
    for sid in x + y:
        pool.release(0, sid, keep_cached=True)
    _, ev = pool.alloc_evict(1, 3)
    assert sorted(ev) == [(0, s) for s in y]          # page 1 (latest access 5) goes before page 0 (9)


@pytest.mark.parametrize("seed,sizes,n_large", [(1, [256, 384], 12), (2, [2048, 3072, 6144], 10), (3, [64, 640], 30)])
def test_reduces_to_three_steps_when_nothing_is_cached(seed, sizes, n_large):
    L = lcm_bytes(sizes)
    plain = OraclePool(n_large * L, sizes)
    caching = OracleCachingPool(n_large * L, sizes)
    h2, refs = {}, {}
    for op in scripts.lowlevel_trace(len(sizes), 6, 1500, seed):
        if op[0] == "alloc":
            _, h, k, req = op
            try:
                want = plain.alloc(k, req)
            except OutOfPages:
                with pytest.raises(OutOfPages):
                    caching.alloc_evict(k, req)
                refs[h] = 0
                continue
            assert caching.alloc_evict(k, req) == (want, [])
            h2[h], refs[h] = (k, want), 1
        elif op[0] == "ref" and refs.get(op[1], 0) > 0:
            plain.ref(*h2[op[1]]); caching.ref(*h2[op[1]]); refs[op[1]] += 1
        elif op[0] == "unref" and refs.get(op[1], 0) > 0:
            plain.free(*h2[op[1]]); caching.free(*h2[op[1]]); refs[op[1]] -= 1
    assert caching.free_large() == caching.n_large


@pytest.mark.parametrize("seed", [4, 5, 6])
def test_invariants_with_caching(seed):
    sizes = [256, 384]
    pool = OracleCachingPool(10 * 768, sizes)
    rng = np.random.default_rng(seed)
    used, cached = [], []
    clock = 0
    for _ in range(1500):
        clock += 1
        u = rng.random()
        if u < 0.5 or not used:
            k, req = int(rng.integers(2)), int(rng.integers(5)) + 1
            try:
                sid, ev = pool.alloc_evict(k, req)
            except OutOfPages:
                assert not cached or all(c[0] != k for c in cached)
                continue
            for e in ev:
                cached.remove(e)
            assert (k, sid) not in used
            used.append((k, sid))
            pool.set_last_access(k, sid, clock)
        elif u < 0.8:
            k, sid = used.pop(int(rng.integers(len(used))))
            keep = bool(rng.random() < 0.7)
            pool.release(k, sid, keep_cached=keep)
            if keep:
                cached.append((k, sid))
        elif cached:
            k, sid = cached.pop(int(rng.integers(len(cached))))
            pool.acquire(k, sid)
            used.append((k, sid))
        # states agree with the bookkeeping of this test
        for k, sid in used:
            assert pool.state(k, sid) == USED
        for k, sid in cached:
            assert pool.state(k, sid) == EVICTABLE
        # no two pages with contents overlap; each lies in a large page of its own kind
        ext = sorted(pool.live_extents())
        assert len(ext) == len(used) + len(cached)
        for (b0, e0, _, _), (b1, e1, _, _) in zip(ext, ext[1:]):
            assert e0 <= b1
        for b, e, k, sid in ext:
            assert pool.large_owner(b // pool.large_bytes)[0] == k
        owned = sum(pool.owned_large(k) for k in range(2))
        assert owned == len({b // pool.large_bytes for b, _, _, _ in ext})
    for k, sid in used:
        pool.release(k, sid, keep_cached=False)
    while cached:
        k, sid = cached.pop()
        pool.acquire(k, sid)
        pool.release(k, sid, keep_cached=False)
    assert pool.free_large() == pool.n_large


def test_state_errors():
    pool = OracleCachingPool(4 * 768, [256, 384])
    a = pool.alloc(0, 1)
    with pytest.raises(InvalidOp):
        pool.acquire(0, a)                       # used, not evictable
    pool.release(0, a, keep_cached=True)
    with pytest.raises(InvalidOp):
        pool.release(0, a, keep_cached=True)     # not in use
    pool.acquire(0, a)
    pool.release(0, a, keep_cached=False)
    assert pool.state(0, a) == EMPTY
    with pytest.raises(InvalidOp):
        pool.set_last_access(0, a, 3)
    with pytest.raises(InvalidOp):
        pool.acquire(0, a)


# ------------------------------------------------------------------- hit rules (Sec. 5.2, 5.3)
def test_hit_rule_example_of_the_paper():
    g = GOLD["hit_rule"]
    req = g["request"]
    # The cache-state figure is not in the text; these states are the ones the printed prefix
    # sets imply: self-attention has A..I cached; a window of 2 (ABC is invalid "because both B
    # and C must remain cached") has exactly C, D, H, I, J cached.
    full_hit = [ch in "ABCDEFGHI" for ch in req]
    win_hit = [ch in "CDHIJ" for ch in req]
    full = possible_prefixes_full(full_hit)
    win = possible_prefixes_window(win_hit, 2)
    assert [req[:p] for p in full] == [req[:p] for p in range(1, len(g["full_valid_max"]) + 1)]
    assert [req[:p] for p in win] == g["window_valid"]
    for bad in g["window_invalid"]:
        assert len(bad) not in win
    assert longest_common_prefix([full, win]) == len("ABCDEFGHI")


def test_hit_rules_properties():
    rng = np.random.default_rng(0)
    for _ in range(50):
        n = int(rng.integers(1, 40))
        hit = (rng.random(n) < 0.8).tolist()
        full = possible_prefixes_full(hit)
        assert full == list(range(1, (hit.index(False) if False in hit else n) + 1))
        # a window at least as long as the request is the full rule; window 1 = "last token cached"
        assert possible_prefixes_window(hit, n) == full
        assert possible_prefixes_window(hit, 1) == [p for p in range(1, n + 1) if hit[p - 1]]
        for w in (2, 3, 7):
            wv = possible_prefixes_window(hit, w)
            assert set(full) <= set(wv)              # the window rule is never stricter
            for p in wv:
                assert all(hit[max(0, p - w):p])
    stride = GOLD["mamba_stride"]["stride"]
    hit = [False] * 2000
    hit[511] = hit[1535] = True
    assert possible_prefixes_every(hit, stride) == [512, 1536]
    assert longest_common_prefix([[1, 2, 3], [5, 6]]) == 0
    assert longest_common_prefix([list(range(1, 1600)), [512, 1536], [4, 512, 600]]) == 512
