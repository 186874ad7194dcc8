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
