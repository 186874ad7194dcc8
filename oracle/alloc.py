"""Allocator oracle: the two-level LCM allocator, written out step by step.

TEST INFRASTRUCTURE ONLY (see the package docstring).  Slow on purpose: every
decision is a linear scan in page-number order so it can be checked by eye.

What it follows
  * Sec. 1 / Sec. 4.1: the pool is cut into equal large pages whose size is the
    least common multiple of the per-layer-type small-page sizes (2 KB, 3 KB ->
    6 KB; 256, 384 -> 768).  A large page handed to a layer type is split into
    large/small_k small pages of that type.
  * Sec. 4.1 allocate()/free(): a small page is taken from a large page of that
    type; when none has room a new large page is requested and split; when all
    small pages of a large page are unused the large page goes back.
  * Sec. 4.3: every large page, with all its small pages, is associated with
    one request; allocation tries (1) an unused small page associated with the
    asking request, (2) a fresh large page, which becomes associated with the
    asking request, (3) an unused small page of this type associated with
    another request.
  * Sec. 4.1 last paragraph / Sec. 4.2: a type's pages are named by small-page
    ids of that type, id * small_page_bytes being the byte offset from the
    common pool base (text pages P2, P3 lie inside large page 1 when a large
    page holds two of them).
  * Sec. 5.1 (sliding window): only the last `window` tokens are needed, so a
    page wholly left of the window can be freed.

Readings where the paper is silent (each is a contract of this build, not of
the paper; tests assert the paper-mandated invariants separately from these):
  * ties: the lowest-numbered eligible large page, and inside it the lowest
    free slot; step 2 takes the lowest-numbered free large page;
  * a large page keeps its request association until it is returned, even if
    only slots taken by other requests (step 3) keep it alive;
  * a large page is returned inside the free() call that empties it;
  * prefix sharing is a reference count per small page: free() drops one
    reference and the slot becomes unused at zero;
  * the window contains the token being decoded: with L tokens cached after
    the append, tokens [L-W, L) are needed (Fig. last-access: window 2,
    "DE->F").
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np


class OutOfPages(Exception):
    """No small page can be produced by steps 1-3 (no eviction on this path)."""


class InvalidOp(Exception):
    """Bad kind / id, double free, ref of an unused page, bad geometry."""


def lcm_bytes(sizes: Sequence[int]) -> int:
    """Compatible page size of Sec. 1 / Sec. 4.1: lcm of all small-page sizes."""
    out = 1
    for s in sizes:
        if s <= 0:
            raise InvalidOp("small page size must be positive")
        out = out * s // math.gcd(out, s)
    return out


def kv_small_page_bytes(n_layers: int, n_kv_heads: int, head_dim: int,
                        tokens_per_page: int, elem_bytes: int) -> int:
    """Small-page size of an attention layer type (Sec. 4.1 footnote, Sec. 4.2).

    Per token and layer the cache holds one K and one V vector per KV head;
    a small page holds tokens_per_page tokens for *all* layers of the type
    (128 x 2 cross layers = 256, 128 x 3 self layers = 384 in the footnote).
    """
    per_token_per_layer = 2 * n_kv_heads * head_dim * elem_bytes
    return per_token_per_layer * n_layers * tokens_per_page


class OraclePool:
    """Level 1 (large pages) and level 2 (per-type small pages) of Sec. 4.1.

    policy = "request_aware": steps 1-3 of Sec. 4.3.
    policy = "naive": the strategy Sec. 4.3 argues against (Fig. internal_frag
    a): lowest free slot of the type regardless of request, else a new large
    page.  Kept only so a test can show the difference the paper describes.
    """

    def __init__(self, pool_bytes: int, small_page_bytes: Sequence[int],
                 large_page_bytes: Optional[int] = None,
                 policy: str = "request_aware"):
        if policy not in ("request_aware", "naive"):
            raise InvalidOp("unknown policy")
        self.S = [int(s) for s in small_page_bytes]
        if not self.S:
            raise InvalidOp("no kinds")
        lcm = lcm_bytes(self.S)
        self.large_bytes = lcm if large_page_bytes is None else int(large_page_bytes)
        if self.large_bytes <= 0 or self.large_bytes % lcm != 0:
            raise InvalidOp("large page must be a common multiple of all small pages")
        self.n_large = int(pool_bytes) // self.large_bytes
        self.r = [self.large_bytes // s for s in self.S]       # small pages per large page
        self.policy = policy
        # level 1: which kind owns each large page (-1: free), and for which request
        self.large_kind = np.full(self.n_large, -1, dtype=np.int64)
        self.large_req = np.zeros(self.n_large, dtype=np.int64)
        # level 2: reference count of every small page of every kind (0: unused)
        self.refcount = [np.zeros(self.n_large * rk, dtype=np.int64) for rk in self.r]

    # ---- helpers -------------------------------------------------------
    def _check_kind(self, k: int) -> None:
        if not (0 <= k < len(self.S)):
            raise InvalidOp("bad kind")

    def _slots(self, k: int, large: int) -> np.ndarray:
        rk = self.r[k]
        return self.refcount[k][large * rk:(large + 1) * rk]

    def _take_lowest_free_slot(self, k: int, large: int) -> int:
        slots = self._slots(k, large)
        slot = int(np.flatnonzero(slots == 0)[0])
        sid = large * self.r[k] + slot
        self.refcount[k][sid] = 1
        return sid

    def _larges_with_room(self, k: int, mask: np.ndarray) -> np.ndarray:
        """Large pages selected by mask, owned by kind k, with an unused slot."""
        rk = self.r[k]
        unused = (self.refcount[k].reshape(self.n_large, rk) == 0).any(axis=1)
        return np.flatnonzero(mask & (self.large_kind == k) & unused)

    # ---- Sec. 4.1 allocate() with the order of Sec. 4.3 ------------------
    def alloc(self, k: int, request: int) -> int:
        self._check_kind(k)
        everyone = np.ones(self.n_large, dtype=bool)
        if self.policy == "request_aware":
            # step 1: an unused small page associated with this request
            mine = self._larges_with_room(k, self.large_req == request)
            if mine.size:
                return self._take_lowest_free_slot(k, int(mine[0]))
        else:
            anyone = self._larges_with_room(k, everyone)
            if anyone.size:
                return self._take_lowest_free_slot(k, int(anyone[0]))
        # step 2: a new large page, all of whose small pages join this request
        free_large = np.flatnonzero(self.large_kind == -1)
        if free_large.size:
            large = int(free_large[0])
            self.large_kind[large] = k
            self.large_req[large] = request
            return self._take_lowest_free_slot(k, large)
        # step 3: an unused small page of this type associated with another request
        anyone = self._larges_with_room(k, everyone)
        if anyone.size:
            return self._take_lowest_free_slot(k, int(anyone[0]))
        raise OutOfPages(f"kind {k}")

    def ref(self, k: int, sid: int) -> None:
        self._check_kind(k)
        if not (0 <= sid < self.refcount[k].size) or self.refcount[k][sid] == 0:
            raise InvalidOp("ref of an unused small page")
        self.refcount[k][sid] += 1

    # ---- Sec. 4.1 free(small_page_id) ------------------------------------
    def free(self, k: int, sid: int) -> None:
        self._check_kind(k)
        if not (0 <= sid < self.refcount[k].size) or self.refcount[k][sid] == 0:
            raise InvalidOp("free of an unused small page")
        self.refcount[k][sid] -= 1
        large = sid // self.r[k]
        if not self._slots(k, large).any():          # every small page unused
            self.large_kind[large] = -1              # back to the large-page allocator
            self.large_req[large] = 0

    # ---- addressing (Sec. 4.1 last paragraph, Sec. 4.2) -------------------
    def byte_offset(self, k: int, sid: int) -> int:
        self._check_kind(k)
        return sid * self.S[k]

    # ---- accounting -------------------------------------------------------
    def free_large(self) -> int:
        return int((self.large_kind == -1).sum())

    def owned_large(self, k: int) -> int:
        return int((self.large_kind == k).sum())

    def used_small(self, k: int) -> int:
        return int((self.refcount[k] > 0).sum())

    def unused_small_in_owned(self, k: int) -> int:
        """Small pages lost to internal fragmentation (Sec. 4.3, Sec. 4.4)."""
        return self.owned_large(k) * self.r[k] - self.used_small(k)

    def used_bytes(self) -> int:
        return sum(self.used_small(k) * self.S[k] for k in range(len(self.S)))

    def live_extents(self) -> List[Tuple[int, int, int, int]]:
        """(byte_begin, byte_end, kind, id) of every live small page."""
        out = []
        for k in range(len(self.S)):
            for sid in np.flatnonzero(self.refcount[k] > 0):
                b = int(sid) * self.S[k]
                out.append((b, b + self.S[k], k, int(sid)))
        return out

    def large_owner(self, large: int) -> Tuple[int, int]:
        return int(self.large_kind[large]), int(self.large_req[large])


def first_needed_token(seq_len: int, window: int) -> int:
    """First token a layer still needs once seq_len tokens are cached.

    Full attention needs every token; a sliding-window layer (Sec. 3.1 a,
    Sec. 5.1) needs the last `window` ones, the newest included.
    """
    if window <= 0:
        return 0
    return max(0, seq_len - window)


class OracleRequests:
    """Per request and kind: the list of small-page ids, by logical page.

    This is the "attention metadata per layer type" of Sec. 4.2 item (2): row
    b of kind k's block table is the list kept here, -1 where a page is not
    resident (never allocated, or a window page that slid out).
    """

    def __init__(self, pool: OraclePool, tokens_per_page: Sequence[int],
                 window: Sequence[int]):
        self.pool = pool
        self.T = list(tokens_per_page)
        self.W = list(window)
        self.pages: Dict[Tuple[int, int], List[int]] = {}

    def extend(self, request: int, k: int, new_len: int) -> None:
        """Make kind k of `request` hold tokens [0, new_len).

        New logical pages are allocated in order; then every resident page that
        lies wholly before the first needed token is freed and its entry
        becomes -1 (Sec. 5.1: tokens outside the window are not needed).
        """
        T = self.T[k]
        lst = self.pages.setdefault((request, k), [])
        need = -(-new_len // T)
        while len(lst) < need:
            lst.append(self.pool.alloc(k, request))
        lo = first_needed_token(new_len, self.W[k])
        for p in range(len(lst)):
            if T * (p + 1) <= lo and lst[p] >= 0:
                self.pool.free(k, lst[p])
                lst[p] = -1

    def share_prefix(self, src: int, dst: int, k: int, n_pages: int) -> None:
        """dst starts as a sharer of src's first n_pages pages (refcount + 1)."""
        s = self.pages.get((src, k), [])
        if (dst, k) in self.pages and self.pages[(dst, k)]:
            raise InvalidOp("destination already has pages")
        if n_pages > len(s):
            raise InvalidOp("source has fewer pages")
        d = []
        for p in range(n_pages):
            if s[p] >= 0:
                self.pool.ref(k, s[p])
            d.append(s[p])
        self.pages[(dst, k)] = d

    def free_request(self, request: int) -> None:
        for (r, k) in sorted(self.pages):
            if r != request:
                continue
            for sid in self.pages[(r, k)]:
                if sid >= 0:
                    self.pool.free(k, sid)
        for key in [key for key in self.pages if key[0] == request]:
            del self.pages[key]

    def row(self, request: int, k: int, width: int) -> List[int]:
        lst = self.pages.get((request, k), [])
        if len(lst) > width:
            raise InvalidOp("row wider than the table")
        return lst + [-1] * (width - len(lst))


# ---------------------------------------------------------------------------
# Sec. 5: page states, LRU keys and the five-step allocation of Sec. 5.4
# ---------------------------------------------------------------------------
EMPTY, EVICTABLE, USED = 0, 1, 2


class OracleCachingPool(OraclePool):
    """The allocator with prefix-cache page states (Sec. 5.4) and LRU eviction (Sec. 5.1).

    A small page is empty (no valid KV), evictable (valid KV, used by no request) or used.
    release(keep_cached=True) leaves a page evictable instead of empty; acquire() takes an
    evictable page back into use (a prefix-cache hit).  Allocation follows the five steps of
    Sec. 5.4; with no evictable page anywhere they reduce to the three steps of Sec. 4.3.

    LRU keys per small page: last_access (Sec. 5.1 update_last_access) and prefix_length
    (Sec. 5.1 set_prefix_length).  The page with the earliest last access goes first; among
    equal times the one with the largest prefix length (Sec. 5.1: "the token with the highest
    length is evicted before other tokens").

    A large page is evictable when all its small pages are evictable (Sec. 5.4): one used or
    one empty small page keeps it out of step 3.  Its LRU time is the latest last access among
    all its small pages (Sec. 5.4, step 3).

    Readings where the paper is silent:
      * ties between large pages of equal LRU time go to the larger maximum prefix length
        (Sec. 5.1 states the rule for tokens), then to the lower page number;
      * remaining ties between small pages go to the lower id.
    """

    def __init__(self, *args, **kwargs):
        super().__init__(*args, **kwargs)
        self.cached = [np.zeros(self.n_large * rk, dtype=bool) for rk in self.r]
        self.last_access = [np.zeros(self.n_large * rk, dtype=np.int64) for rk in self.r]
        self.prefix_length = [np.zeros(self.n_large * rk, dtype=np.int64) for rk in self.r]

    # ---- states -----------------------------------------------------------
    def state(self, k: int, sid: int) -> int:
        if self.refcount[k][sid] > 0:
            return USED
        return EVICTABLE if self.cached[k][sid] else EMPTY

    def _empty_mask(self, k: int) -> np.ndarray:
        return (self.refcount[k] == 0) & ~self.cached[k]

    def _larges_with_empty(self, k: int, mask: np.ndarray) -> np.ndarray:
        has = self._empty_mask(k).reshape(self.n_large, self.r[k]).any(axis=1)
        return np.flatnonzero(mask & (self.large_kind == k) & has)

    def _take_lowest_empty(self, k: int, large: int) -> int:
        rk = self.r[k]
        slot = int(np.flatnonzero(self._empty_mask(k)[large * rk:(large + 1) * rk])[0])
        sid = large * rk + slot
        self.refcount[k][sid] = 1
        return sid

    def set_last_access(self, k: int, sid: int, time: int) -> None:
        self._check_kind(k)
        if self.state(k, sid) == EMPTY:
            raise InvalidOp("empty page has no access time")
        self.last_access[k][sid] = time

    def set_prefix_length(self, k: int, sid: int, length: int) -> None:
        self._check_kind(k)
        if self.state(k, sid) == EMPTY:
            raise InvalidOp("empty page has no prefix length")
        self.prefix_length[k][sid] = length

    def release(self, k: int, sid: int, keep_cached: bool) -> None:
        """One reference fewer; at zero the page becomes evictable (keep_cached) or empty."""
        self._check_kind(k)
        if not (0 <= sid < self.refcount[k].size) or self.refcount[k][sid] == 0:
            raise InvalidOp("release of a page that is not in use")
        self.refcount[k][sid] -= 1
        if self.refcount[k][sid] == 0:
            self.cached[k][sid] = bool(keep_cached)
            self._return_large_if_empty(k, sid // self.r[k])

    def free(self, k: int, sid: int) -> None:      # Sec. 4.1 free(): no caching
        self.release(k, sid, keep_cached=False)

    def acquire(self, k: int, sid: int) -> None:
        """Prefix-cache hit: an evictable page is used again."""
        self._check_kind(k)
        if not (0 <= sid < self.refcount[k].size) or self.state(k, sid) != EVICTABLE:
            raise InvalidOp("acquire of a page that is not evictable")
        self.cached[k][sid] = False
        self.refcount[k][sid] = 1

    def _return_large_if_empty(self, k: int, large: int) -> None:
        rk = self.r[k]
        sl = slice(large * rk, (large + 1) * rk)
        if not self.refcount[k][sl].any() and not self.cached[k][sl].any():
            self.large_kind[large] = -1
            self.large_req[large] = 0

    # ---- Sec. 5.4: the five steps -------------------------------------------
    def alloc_evict(self, k: int, request: int):
        """Returns (small id, [(kind, id) of every page evicted to make room])."""
        self._check_kind(k)
        # 1. an empty small page associated with this request
        mine = self._larges_with_empty(k, self.large_req == request)
        if mine.size:
            return self._take_lowest_empty(k, int(mine[0])), []
        # 2. an empty large page
        free_large = np.flatnonzero(self.large_kind == -1)
        if free_large.size:
            large = int(free_large[0])
            self.large_kind[large] = k
            self.large_req[large] = request
            return self._take_lowest_empty(k, large), []
        # 3. evict an evictable large page, least recently used first
        best, best_key = None, None
        for large in range(self.n_large):
            ko = int(self.large_kind[large])
            if ko < 0:
                continue
            rk = self.r[ko]
            ids = np.arange(large * rk, (large + 1) * rk)
            if not self.cached[ko][ids].all():       # evictable = every small page evictable
                continue
            key = (int(self.last_access[ko][ids].max()), -int(self.prefix_length[ko][ids].max()), large)
            if best_key is None or key < best_key:
                best, best_key = large, key
        if best is not None:
            ko = int(self.large_kind[best])
            rk = self.r[ko]
            evicted = [(ko, int(s)) for s in range(best * rk, (best + 1) * rk)]
            for _, s in evicted:
                self.cached[ko][s] = False           # "all small pages ... are marked empty"
            self.large_kind[best] = k            # all its small pages are empty now: re-typed
            self.large_req[best] = request
            return self._take_lowest_empty(k, best), evicted
        # 4. an empty small page of this kind associated with another request
        anyone = self._larges_with_empty(k, np.ones(self.n_large, dtype=bool))
        if anyone.size:
            return self._take_lowest_empty(k, int(anyone[0])), []
        # 5. evict an evictable small page of this kind, least recently used first
        cand = np.flatnonzero(self.cached[k] & (self.refcount[k] == 0))
        if cand.size:
            keys = [(int(self.last_access[k][s]), -int(self.prefix_length[k][s]), int(s)) for s in cand]
            sid = min(keys)[2]
            self.cached[k][sid] = False
            self.refcount[k][sid] = 1
            return sid, [(k, sid)]
        raise OutOfPages(f"kind {k}")

    def alloc(self, k: int, request: int) -> int:
        return self.alloc_evict(k, request)[0]

    def evictable_small(self, k: int) -> int:
        return int((self.cached[k] & (self.refcount[k] == 0)).sum())

    def live_extents(self):
        out = super().live_extents()
        for k in range(len(self.S)):
            for sid in np.flatnonzero(self.cached[k] & (self.refcount[k] == 0)):
                b = int(sid) * self.S[k]
                out.append((b, b + self.S[k], k, int(sid)))
        return out


# ---------------------------------------------------------------------------
# Sec. 5.2 / 5.3: customised hit rules
# ---------------------------------------------------------------------------
def possible_prefixes_full(is_hit: Sequence[bool]) -> List[int]:
    """Full attention: a prefix is valid when every token in it is cached (Sec. 5.2)."""
    out = []
    for p in range(1, len(is_hit) + 1):
        if not is_hit[p - 1]:
            break
        out.append(p)
    return out


def possible_prefixes_window(is_hit: Sequence[bool], window: int) -> List[int]:
    """Sliding window: prefix p is valid when its last `window` tokens are cached
    (Fig. interface/sliding: all x in [0, sliding) with is_hit[p - x], token indices from 1)."""
    out = []
    for p in range(1, len(is_hit) + 1):
        if all(is_hit[p - x - 1] for x in range(window) if p - x >= 1):
            out.append(p)
    return out


def possible_prefixes_every(is_hit: Sequence[bool], stride: int) -> List[int]:
    """State-space layers cache one state every `stride` tokens (512 in Sec. 5.3): prefix p
    is valid when p is a multiple of the stride and the state after token p is cached."""
    return [p for p in range(stride, len(is_hit) + 1, stride) if is_hit[p - 1]]


def longest_common_prefix(valid_sets: Sequence[Sequence[int]]) -> int:
    """Sec. 5.2: the longest prefix valid for every layer type (0 when there is none)."""
    common = set(valid_sets[0])
    for v in valid_sets[1:]:
        common &= set(v)
    return max(common) if common else 0
