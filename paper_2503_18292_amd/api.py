"""Python names for the C ABI of include/jenga.h (argument marshalling only).

Device arguments are torch tensors on the GPU (used as raw pointers); kernels are
enqueued on torch's current stream.  Every status other than JENGA_OK raises JengaError.
"""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence

from . import _lib
from ._lib import KindDesc, KindStats, PoolInfo

F32, BF16 = 0, 1
FULL, WINDOW, CROSS, OPAQUE = 0, 1, 2, 3

STATUS_NAMES = {-1: "INVALID", -2: "OOM", -3: "ALIGN", -4: "WORKSPACE", -5: "HIP", -6: "UNSUPPORTED"}


class JengaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        msg = _lib.load().jenga_strerror(int(status)).decode()
        super().__init__(f"{where}: {STATUS_NAMES.get(int(status), status)} ({msg})")


def _check(status: int, where: str) -> int:
    if status < 0:
        raise JengaError(status, where)
    return status


def _ptr(t) -> Optional[int]:
    """Raw address of a torch tensor (or None)."""
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream() -> Optional[int]:
    import torch
    return torch.cuda.current_stream().cuda_stream or None


def _desc_array(kinds: Sequence[KindDesc]):
    arr = (KindDesc * len(kinds))()
    for i, k in enumerate(kinds):
        arr[i] = k
    return arr


def make_kind(type: int, dtype: int = BF16, n_layers: int = 1, n_kv_heads: int = 0, head_dim: int = 0,
              tokens_per_page: Optional[int] = None, window: int = 0, small_page_bytes: int = 0) -> KindDesc:
    if tokens_per_page is None:                 # an OPAQUE page is one unit; attention pages default to 16 tokens
        tokens_per_page = 1 if type == OPAQUE else 16
    return KindDesc(type, dtype, n_layers, n_kv_heads, head_dim, tokens_per_page, window, 0,
                    small_page_bytes)


def lcm_page_bytes(kinds: Sequence[KindDesc]) -> int:
    out = C.c_int64(0)
    _check(_lib.load().jenga_lcm_page_bytes(_desc_array(kinds), len(kinds), C.byref(out)),
           "jenga_lcm_page_bytes")
    return out.value


def possible_prefixes(rule: int, param: int, is_hit) -> list:
    """Valid prefix lengths for one layer type (jenga_possible_prefixes)."""
    n = len(is_hit)
    hit = (C.c_uint8 * max(n, 1))(*[1 if h else 0 for h in is_hit])
    out = (C.c_uint8 * (n + 1))()
    _check(_lib.load().jenga_possible_prefixes(rule, param, hit, n, out), "jenga_possible_prefixes")
    return [p for p in range(1, n + 1) if out[p]]


def longest_common_prefix(valid_sets, n_tokens: int) -> int:
    arrs = []
    for v in valid_sets:
        a = (C.c_uint8 * (n_tokens + 1))()
        for p in v:
            a[p] = 1
        arrs.append(a)
    ptrs = (C.c_void_p * len(arrs))(*[C.cast(a, C.c_void_p) for a in arrs])
    return _check(_lib.load().jenga_longest_common_prefix(ptrs, len(arrs), n_tokens),
                  "jenga_longest_common_prefix")


HIT_FULL, HIT_WINDOW, HIT_EVERY = 0, 1, 2
PAGE_EMPTY, PAGE_EVICTABLE, PAGE_USED = 0, 1, 2


def version() -> int:
    return _lib.load().jenga_version()


def stream_copy(dst, src, nbytes: int) -> None:
    _check(_lib.load().jenga_stream_copy(_ptr(dst), _ptr(src), nbytes, _stream()), "jenga_stream_copy")


def stream_read(src, nbytes: int, sink) -> None:
    _check(_lib.load().jenga_stream_read(_ptr(src), nbytes, _ptr(sink), _stream()), "jenga_stream_read")


class Pool:
    """jenga_pool handle; method names follow the C entry points without the prefix."""

    def __init__(self, device_base: Optional[int], pool_bytes: int, kinds: Sequence[KindDesc],
                 large_page_bytes: Optional[int] = None):
        self._lib = _lib.load()
        self.kinds = list(kinds)
        if large_page_bytes is None:
            large_page_bytes = lcm_page_bytes(kinds)
        handle = C.c_void_p()
        _check(self._lib.jenga_pool_create(device_base, pool_bytes, large_page_bytes,
                                           _desc_array(kinds), len(kinds), C.byref(handle)),
               "jenga_pool_create")
        self._h = handle

    def destroy(self) -> None:
        if self._h:
            self._lib.jenga_pool_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # ---- host: allocator ------------------------------------------------------
    def alloc_small(self, kind: int, request: int) -> int:
        out = C.c_int32(-1)
        _check(self._lib.jenga_alloc_small(self._h, kind, request, C.byref(out)), "jenga_alloc_small")
        return out.value

    def ref_small(self, kind: int, small_id: int) -> None:
        _check(self._lib.jenga_ref_small(self._h, kind, small_id), "jenga_ref_small")

    def free_small(self, kind: int, small_id: int) -> None:
        _check(self._lib.jenga_free_small(self._h, kind, small_id), "jenga_free_small")

    # ---- host: prefix-cache side ----------------------------------------------------
    def alloc_small_evict(self, kind: int, request: int, capacity: int = 256):
        """Returns (small id, [(kind, id) of every page evicted to make room])."""
        out, n = C.c_int32(-1), C.c_int32(0)
        ks, ids = (C.c_int32 * capacity)(), (C.c_int32 * capacity)()
        _check(self._lib.jenga_alloc_small_evict(self._h, kind, request, C.byref(out), ks, ids, capacity,
                                                 C.byref(n)), "jenga_alloc_small_evict")
        return out.value, [(ks[i], ids[i]) for i in range(min(n.value, capacity))]

    def release_small(self, kind: int, small_id: int, keep_cached: bool) -> None:
        _check(self._lib.jenga_release_small(self._h, kind, small_id, int(keep_cached)), "jenga_release_small")

    def acquire_cached(self, kind: int, small_id: int) -> None:
        _check(self._lib.jenga_acquire_cached(self._h, kind, small_id), "jenga_acquire_cached")

    def set_last_access(self, kind: int, small_id: int, time: int) -> None:
        _check(self._lib.jenga_set_last_access(self._h, kind, small_id, time), "jenga_set_last_access")

    def set_prefix_length(self, kind: int, small_id: int, length: int) -> None:
        _check(self._lib.jenga_set_prefix_length(self._h, kind, small_id, length), "jenga_set_prefix_length")

    def small_state(self, kind: int, small_id: int) -> int:
        out = C.c_int32(0)
        _check(self._lib.jenga_small_state(self._h, kind, small_id, C.byref(out)), "jenga_small_state")
        return out.value

    def request_release(self, request: int, keep_cached: bool) -> None:
        _check(self._lib.jenga_request_release(self._h, request, int(keep_cached)), "jenga_request_release")

    def request_touch(self, request: int, kind: int, first_token: int, end_token: int, time: int) -> None:
        _check(self._lib.jenga_request_touch(self._h, request, kind, first_token, end_token, time),
               "jenga_request_touch")

    def request_set_prefix_lengths(self, request: int, kind: int) -> None:
        _check(self._lib.jenga_request_set_prefix_lengths(self._h, request, kind),
               "jenga_request_set_prefix_lengths")

    def get_info(self) -> PoolInfo:
        out = PoolInfo()
        _check(self._lib.jenga_pool_get_info(self._h, C.byref(out)), "jenga_pool_get_info")
        return out

    def kind_stats(self, kind: int) -> KindStats:
        out = KindStats()
        _check(self._lib.jenga_pool_kind_stats(self._h, kind, C.byref(out)), "jenga_pool_kind_stats")
        return out

    def large_page_owner(self, large_page: int):
        k, r = C.c_int32(0), C.c_int64(0)
        _check(self._lib.jenga_large_page_owner(self._h, large_page, C.byref(k), C.byref(r)),
               "jenga_large_page_owner")
        return k.value, r.value

    def small_refcount(self, kind: int, small_id: int) -> int:
        out = C.c_int32(0)
        _check(self._lib.jenga_small_refcount(self._h, kind, small_id, C.byref(out)),
               "jenga_small_refcount")
        return out.value

    def kv_offset(self, kind: int, small_id: int, layer: int, kv_head: int, is_v: int,
                  token_in_page: int) -> int:
        out = C.c_int64(0)
        _check(self._lib.jenga_kv_offset(self._h, kind, small_id, layer, kv_head, is_v, token_in_page,
                                         C.byref(out)), "jenga_kv_offset")
        return out.value

    # ---- host: requests / block tables ------------------------------------------
    def request_extend(self, request: int, kind: int, new_len: int) -> None:
        _check(self._lib.jenga_request_extend(self._h, request, kind, new_len), "jenga_request_extend")

    def request_share_prefix(self, src: int, dst: int, kind: int, n_pages: int) -> None:
        _check(self._lib.jenga_request_share_prefix(self._h, src, dst, kind, n_pages),
               "jenga_request_share_prefix")

    def request_free(self, request: int) -> None:
        _check(self._lib.jenga_request_free(self._h, request), "jenga_request_free")

    def request_num_pages(self, request: int, kind: int) -> int:
        out = C.c_int32(0)
        _check(self._lib.jenga_request_num_pages(self._h, request, kind, C.byref(out)),
               "jenga_request_num_pages")
        return out.value

    def request_block_table_row(self, request: int, kind: int, width: int) -> List[int]:
        row = (C.c_int32 * max(width, 1))()
        _check(self._lib.jenga_request_block_table_row(self._h, request, kind, row, width),
               "jenga_request_block_table_row")
        return list(row[:width])

    def block_table(self, requests: Sequence[int], kind: int, width: int):
        """Host int32 tensor [len(requests), width] filled row by row by the library."""
        import numpy as np
        import torch
        tab = np.empty((len(requests), max(width, 1)), dtype=np.int32)
        for i, r in enumerate(requests):
            _check(self._lib.jenga_request_block_table_row(
                self._h, r, kind, tab[i].ctypes.data_as(C.POINTER(C.c_int32)), width),
                "jenga_request_block_table_row")
        return torch.from_numpy(tab)

    def requests_extend(self, kind: int, requests, new_lens) -> None:
        """requests, new_lens: contiguous int64 numpy arrays of equal length."""
        _check(self._lib.jenga_requests_extend(self._h, kind, requests.ctypes.data, new_lens.ctypes.data,
                                               len(requests)), "jenga_requests_extend")

    def block_table_fill(self, kind: int, requests, table) -> None:
        """requests: int64 numpy array [n]; table: host int32 torch tensor [n, width], filled in place."""
        _check(self._lib.jenga_block_table_fill(self._h, kind, requests.ctypes.data, len(requests),
                                                table.data_ptr(), table.shape[1]),
               "jenga_block_table_fill")

    # aliases so a script runner can drive the library and the oracle alike
    extend = request_extend
    share_prefix = request_share_prefix
    free_request = request_free

    # ---- device ----------------------------------------------------------------
    def kv_append(self, kind: int, layer: int, k_new, v_new, block_table, seq_lens) -> None:
        _check(self._lib.jenga_kv_append(self._h, kind, layer, _ptr(k_new), _ptr(v_new),
                                         _ptr(block_table), block_table.shape[1], _ptr(seq_lens),
                                         seq_lens.shape[0], _stream()), "jenga_kv_append")

    def kv_write_range(self, kind: int, layer: int, k_src, v_src, cu_tokens, start_pos, block_table) -> None:
        _check(self._lib.jenga_kv_write_range(self._h, kind, layer, _ptr(k_src), _ptr(v_src),
                                              _ptr(cu_tokens), _ptr(start_pos), _ptr(block_table),
                                              block_table.shape[1], start_pos.shape[0], k_src.shape[0],
                                              _stream()), "jenga_kv_write_range")

    def decode_num_partitions(self, kind: int, n_q_heads: int, batch: int, max_seq_len: int,
                              window: int = 0, pages_per_split: int = 0) -> int:
        return _check(self._lib.jenga_decode_num_partitions(self._h, kind, n_q_heads, batch, max_seq_len,
                                                            window, pages_per_split),
                      "jenga_decode_num_partitions")

    def decode_workspace_bytes(self, kind: int, n_q_heads: int, batch: int, max_seq_len: int,
                               window: int = 0, pages_per_split: int = 0) -> int:
        return _check(self._lib.jenga_decode_workspace_bytes(self._h, kind, n_q_heads, batch,
                                                             max_seq_len, window, pages_per_split),
                      "jenga_decode_workspace_bytes")

    def paged_decode(self, kind: int, layer: int, q, block_table, seq_lens, max_seq_len: int,
                     window: int, scale: float, workspace, out, pages_per_split: int = 0,
                     k_new=None, v_new=None) -> None:
        _check(self._lib.jenga_paged_decode(
            self._h, kind, layer, _ptr(q), q.shape[1], _ptr(k_new), _ptr(v_new),
            _ptr(block_table), block_table.shape[1],
            _ptr(seq_lens), seq_lens.shape[0], max_seq_len, window, scale, pages_per_split,
            _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(out), _stream()),
            "jenga_paged_decode")

    def paged_decode_static(self, kind: int, layer: int, q, block_table, seq_lens, max_seq_len: int,
                            window: int, scale: float, out, pages_per_split: int = 0,
                            k_new=None, v_new=None) -> None:
        """jenga_paged_decode with the library's own scratch buffer: allocates nothing."""
        _check(self._lib.jenga_paged_decode_static(
            self._h, kind, layer, _ptr(q), q.shape[1], _ptr(k_new), _ptr(v_new),
            _ptr(block_table), block_table.shape[1],
            _ptr(seq_lens), seq_lens.shape[0], max_seq_len, window, scale, pages_per_split,
            _ptr(out), _stream()), "jenga_paged_decode_static")

    def paged_decode_partial(self, kind: int, layer: int, q, block_table, seq_lens, max_seq_len: int,
                             window: int, scale: float, workspace, pages_per_split: int = 0,
                             k_new=None, v_new=None) -> None:
        _check(self._lib.jenga_paged_decode_partial(
            self._h, kind, layer, _ptr(q), q.shape[1], _ptr(k_new), _ptr(v_new),
            _ptr(block_table), block_table.shape[1],
            _ptr(seq_lens), seq_lens.shape[0], max_seq_len, window, scale, pages_per_split,
            _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()),
            "jenga_paged_decode_partial")

    def splitk_reduce(self, kind: int, n_q_heads: int, seq_lens, max_seq_len: int, window: int,
                      workspace, out, pages_per_split: int = 0) -> None:
        _check(self._lib.jenga_splitk_reduce(
            self._h, kind, n_q_heads, _ptr(seq_lens), seq_lens.shape[0], max_seq_len, window,
            pages_per_split, _ptr(workspace), workspace.numel() * workspace.element_size(),
            _ptr(out), _stream()), "jenga_splitk_reduce")
