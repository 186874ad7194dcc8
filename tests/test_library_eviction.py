"""Prefix-cache side of the library (page states, LRU keys, five-step allocation, hit rules)
against the oracle, bit for bit, through the C ABI.  Host only."""
import json
import os

import numpy as np
import pytest

from oracle.alloc import (EMPTY, EVICTABLE, USED, OracleCachingPool, OutOfPages, lcm_bytes,
                          longest_common_prefix, possible_prefixes_every, possible_prefixes_full,
                          possible_prefixes_window)

import paper_2503_18292_amd as J
from paper_2503_18292_amd import api
from paper_2503_18292_amd.api import make_kind

from test_oracle_eviction import (evictable_large_page_beats_another_requests_empty_slot,
                                  run_last_access_example, small_pages_of_equal_age)

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_examples.json")))


class LibAsOracle:
    """The library behind the oracle's method names, so one script can drive both."""

    def __init__(self, pool):
        self.p = pool

    def alloc(self, k, req):
        return self.p.alloc_small(k, req)

    def alloc_evict(self, k, req):
        sid, ev = self.p.alloc_small_evict(k, req)
        return sid, ev

    def release(self, k, sid, keep_cached):
        self.p.release_small(k, sid, keep_cached)

    def acquire(self, k, sid):
        self.p.acquire_cached(k, sid)

    def set_last_access(self, k, sid, t):
        self.p.set_last_access(k, sid, t)

    def set_prefix_length(self, k, sid, n):
        self.p.set_prefix_length(k, sid, n)


def opaque_pool(n_large, sizes):
    return J.Pool(None, n_large * lcm_bytes(sizes), [make_kind(J.OPAQUE, small_page_bytes=s) for s in sizes])


def test_paper_example_eviction_order_matches_oracle():
    ora = OracleCachingPool(12 * 64, [64, 64])
    lib = LibAsOracle(opaque_pool(12, [64, 64]))
    tok_o = run_last_access_example(ora)
    tok_l = run_last_access_example(lib)
    assert tok_o == tok_l
    for _ in range(12):
        assert lib.alloc_evict(0, 99) == ora.alloc_evict(0, 99)
    with pytest.raises(J.JengaError) as e:
        lib.alloc_evict(0, 99)
    assert e.value.status == -2


def test_mixed_large_page_is_not_evicted_as_a_whole():
    """Sec. 5.4: only a large page whose small pages are ALL evictable is taken by step 3.  The same
    calls on oracle and library: ids, eviction reports and out-of-pages events agree."""
    def script(pool):
        out = []
        def go(k, req):
            try:
                out.append(pool.alloc_evict(k, req))
            except (OutOfPages, J.JengaError):
                out.append("oom")
        for k, req in ((0, 1), (0, 1), (0, 2), (1, 3)):
            go(k, req)
        for t, sid in enumerate((0, 1)):
            pool.set_last_access(0, sid, 10 + t)
            pool.release(0, sid, True)
        go(0, 2); go(0, 7); go(1, 8); go(0, 7)          # page 0 = {evictable, evictable, ., .}: step 4, never step 3
        for sid, t in ((2, 3), (3, 4)):
            pool.set_last_access(0, sid, t)
            pool.release(0, sid, True)
        go(1, 8)                                         # now all four are evictable: step 3
        go(0, 9); go(0, 9)
        pool.set_last_access(0, 6, 5)
        pool.release(0, 6, True)
        go(0, 10); go(0, 10)
        return out
    want = script(OracleCachingPool(3 * 1024, [256, 1024]))
    got = script(LibAsOracle(opaque_pool(3, [256, 1024])))
    assert got == want
    assert want[5] == (2, []) and want[6] == "oom" and want[8] == (0, [(0, 0), (0, 1), (0, 2), (0, 3)])


def test_step_order_and_tie_scenarios_match_the_oracle():
    want = evictable_large_page_beats_another_requests_empty_slot(OracleCachingPool(3 * 1024, [256, 1024]))
    got = evictable_large_page_beats_another_requests_empty_slot(LibAsOracle(opaque_pool(3, [256, 1024])))
    assert (got[0], got[1], got[2]) == (want[0], want[1], want[2])
    assert got[3][0] == want[3][0] and sorted(got[3][1]) == sorted(want[3][1])
    want = small_pages_of_equal_age(OracleCachingPool(1024, [256], 1024))
    pool = J.Pool(None, 1024, [make_kind(J.OPAQUE, small_page_bytes=256)], large_page_bytes=1024)
    assert small_pages_of_equal_age(LibAsOracle(pool)) == want


@pytest.mark.parametrize("seed,sizes,n_large", [(1, [256, 384], 10), (2, [64, 64], 24), (3, [2048, 3072, 6144], 8),
                                                (4, [64, 640], 12), (5, [16384, 32768], 9)])
def test_random_caching_traces_match_oracle(seed, sizes, n_large):
    ora = OracleCachingPool(n_large * lcm_bytes(sizes), sizes)
    pool = opaque_pool(n_large, sizes)
    lib = LibAsOracle(pool)
    rng = np.random.default_rng(seed)
    used, cached = [], []
    n_evictions = 0
    for clock in range(1, 4001):
        u = rng.random()
        if u < 0.45 or not used:
            k, req = int(rng.integers(len(sizes))), int(rng.integers(6)) + 1
            try:
                want = ora.alloc_evict(k, req)
            except OutOfPages:
                with pytest.raises(J.JengaError):
                    lib.alloc_evict(k, req)
                continue
            got = lib.alloc_evict(k, req)
            assert got == want, f"op {clock}"
            n_evictions += len(want[1])
            for e in want[1]:
                cached.remove(e)
            used.append((k, want[0]))
            t = int(rng.integers(clock // 8, clock + 1))      # frequent ties
            ora.set_last_access(k, want[0], t); lib.set_last_access(k, want[0], t)
            n = int(rng.integers(1, 6))
            ora.set_prefix_length(k, want[0], n); lib.set_prefix_length(k, want[0], n)
        elif u < 0.75:
            k, sid = used.pop(int(rng.integers(len(used))))
            keep = bool(rng.random() < 0.75)
            ora.release(k, sid, keep); lib.release(k, sid, keep)
            if keep:
                cached.append((k, sid))
        elif u < 0.85 and cached:
            k, sid = cached.pop(int(rng.integers(len(cached))))
            ora.acquire(k, sid); lib.acquire(k, sid)
            used.append((k, sid))
        elif cached:                                       # keys of an evictable page change
            k, sid = cached[int(rng.integers(len(cached)))]
            t = int(rng.integers(0, clock + 1))
            ora.set_last_access(k, sid, t); lib.set_last_access(k, sid, t)
        if clock % 200 == 0:
            assert pool.get_info().free_large_pages == ora.free_large()
            for k in range(len(sizes)):
                st = pool.kind_stats(k)
                assert st.used_small_pages == ora.used_small(k)
                assert st.evictable_small_pages == ora.evictable_small(k)
                assert st.owned_large_pages == ora.owned_large(k)
                for sid in range(ora.refcount[k].size):
                    assert pool.small_state(k, sid) == ora.state(k, sid)
    assert n_evictions > 50


def test_request_level_touch_prefix_and_release():
    K = lambda s: make_kind(J.OPAQUE, small_page_bytes=s)
    kinds = [make_kind(J.FULL, J.BF16, 1, 1, 64, 16), make_kind(J.WINDOW, J.BF16, 1, 1, 64, 16, window=32)]
    pool = J.Pool(None, 64 * J.lcm_page_bytes(kinds), kinds)
    pool.request_extend(1, 0, 100)
    pool.request_extend(1, 1, 100)
    # Sec. 5.1: full attention stamps everything, the window layer only the window
    pool.request_touch(1, 0, 0, 100, 7)
    pool.request_touch(1, 1, 100 - 32, 100, 7)
    pool.request_set_prefix_lengths(1, 0)
    pool.request_set_prefix_lengths(1, 1)
    rows = [pool.request_block_table_row(1, k, 7) for k in (0, 1)]
    assert all(s >= 0 for s in rows[0]) and [s >= 0 for s in rows[1]] == [False] * 4 + [True] * 3
    pool.request_release(1, keep_cached=True)
    assert pool.kind_stats(0).evictable_small_pages == 7 and pool.kind_stats(1).evictable_small_pages == 3
    assert pool.kind_stats(0).used_small_pages == 0
    for sid in rows[0]:
        assert pool.small_state(0, sid) == api.PAGE_EVICTABLE
    # a second request hits the cached prefix of the full kind, then everything is dropped
    for sid in rows[0][:4]:
        pool.acquire_cached(0, sid)
    assert pool.kind_stats(0).used_small_pages == 4
    for sid in rows[0][:4]:
        pool.release_small(0, sid, keep_cached=False)
    for sid in rows[0][4:]:
        pool.acquire_cached(0, sid); pool.free_small(0, sid)
    for sid in rows[1][4:]:
        pool.acquire_cached(1, sid); pool.free_small(1, sid)
    info = pool.get_info()
    assert info.free_large_pages == info.n_large_pages
    with pytest.raises(J.JengaError):
        pool.acquire_cached(0, rows[0][0])
    with pytest.raises(J.JengaError):
        pool.set_last_access(0, rows[0][0], 1)        # empty pages carry no keys


def test_hit_rules_match_oracle_and_paper_example():
    g = GOLD["hit_rule"]
    req = g["request"]
    full = api.possible_prefixes(api.HIT_FULL, 0, [ch in "ABCDEFGHI" for ch in req])
    win = api.possible_prefixes(api.HIT_WINDOW, 2, [ch in "CDHIJ" for ch in req])
    assert [req[:p] for p in win] == g["window_valid"]
    assert full == list(range(1, 10))
    assert api.longest_common_prefix([full, win], len(req)) == 9
    rng = np.random.default_rng(3)
    for _ in range(200):
        n = int(rng.integers(0, 60))
        hit = (rng.random(n) < 0.85).tolist()
        assert api.possible_prefixes(api.HIT_FULL, 0, hit) == possible_prefixes_full(hit)
        w = int(rng.integers(1, 12))
        assert api.possible_prefixes(api.HIT_WINDOW, w, hit) == possible_prefixes_window(hit, w)
        st = int(rng.integers(1, 9))
        assert api.possible_prefixes(api.HIT_EVERY, st, hit) == possible_prefixes_every(hit, st)
        sets = [possible_prefixes_full(hit), possible_prefixes_window(hit, w), possible_prefixes_every(hit, st)]
        if n:
            assert api.longest_common_prefix(sets, n) == longest_common_prefix(sets)
    with pytest.raises(J.JengaError):
        api.possible_prefixes(api.HIT_WINDOW, 0, [True])
    with pytest.raises(J.JengaError):
        api.possible_prefixes(7, 1, [True])
