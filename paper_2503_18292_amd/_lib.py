"""ctypes loader for libjenga.so: declares every entry point of include/jenga.h.

Fails loudly when the library has not been built; there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
# JENGA_LIB lets a developer point the binding at another build of the same library
LIB_PATH = os.environ.get("JENGA_LIB") or os.path.join(HERE, "libjenga.so")

c_i32, c_i64, c_f32, c_vp = C.c_int32, C.c_int64, C.c_float, C.c_void_p
p_i32, p_i64 = C.POINTER(C.c_int32), C.POINTER(C.c_int64)


class KindDesc(C.Structure):
    _fields_ = [("type", c_i32), ("dtype", c_i32), ("n_layers", c_i32), ("n_kv_heads", c_i32),
                ("head_dim", c_i32), ("tokens_per_page", c_i32), ("window", c_i32),
                ("reserved", c_i32), ("small_page_bytes", c_i64)]


class PoolInfo(C.Structure):
    _fields_ = [("large_page_bytes", c_i64), ("n_large_pages", c_i64), ("free_large_pages", c_i64),
                ("n_kinds", c_i32), ("reserved", c_i32)]


class KindStats(C.Structure):
    _fields_ = [("small_page_bytes", c_i64), ("slice_bytes", c_i64), ("small_per_large", c_i64),
                ("owned_large_pages", c_i64), ("used_small_pages", c_i64),
                ("unused_small_pages", c_i64), ("evictable_small_pages", c_i64)]


# name -> (restype, argtypes); mirrors include/jenga.h one to one
SIGNATURES = {
    "jenga_lcm_page_bytes": (C.c_int, [C.POINTER(KindDesc), c_i32, p_i64]),
    "jenga_pool_create": (C.c_int, [c_vp, c_i64, c_i64, C.POINTER(KindDesc), c_i32, C.POINTER(c_vp)]),
    "jenga_pool_destroy": (C.c_int, [c_vp]),
    "jenga_alloc_small": (C.c_int, [c_vp, c_i32, c_i64, p_i32]),
    "jenga_ref_small": (C.c_int, [c_vp, c_i32, c_i32]),
    "jenga_free_small": (C.c_int, [c_vp, c_i32, c_i32]),
    "jenga_pool_get_info": (C.c_int, [c_vp, C.POINTER(PoolInfo)]),
    "jenga_pool_kind_stats": (C.c_int, [c_vp, c_i32, C.POINTER(KindStats)]),
    "jenga_large_page_owner": (C.c_int, [c_vp, c_i64, p_i32, p_i64]),
    "jenga_small_refcount": (C.c_int, [c_vp, c_i32, c_i32, p_i32]),
    "jenga_kv_offset": (C.c_int, [c_vp, c_i32, c_i32, c_i32, c_i32, c_i32, c_i32, p_i64]),
    "jenga_request_extend": (C.c_int, [c_vp, c_i64, c_i32, c_i64]),
    "jenga_request_share_prefix": (C.c_int, [c_vp, c_i64, c_i64, c_i32, c_i32]),
    "jenga_request_free": (C.c_int, [c_vp, c_i64]),
    "jenga_request_num_pages": (C.c_int, [c_vp, c_i64, c_i32, p_i32]),
    "jenga_request_block_table_row": (C.c_int, [c_vp, c_i64, c_i32, p_i32, c_i32]),
    "jenga_requests_extend": (C.c_int, [c_vp, c_i32, c_vp, c_vp, c_i32]),
    "jenga_block_table_fill": (C.c_int, [c_vp, c_i32, c_vp, c_i32, c_vp, c_i32]),
    "jenga_alloc_small_evict": (C.c_int, [c_vp, c_i32, c_i64, p_i32, p_i32, p_i32, c_i32, p_i32]),
    "jenga_release_small": (C.c_int, [c_vp, c_i32, c_i32, c_i32]),
    "jenga_acquire_cached": (C.c_int, [c_vp, c_i32, c_i32]),
    "jenga_set_last_access": (C.c_int, [c_vp, c_i32, c_i32, c_i64]),
    "jenga_set_prefix_length": (C.c_int, [c_vp, c_i32, c_i32, c_i64]),
    "jenga_small_state": (C.c_int, [c_vp, c_i32, c_i32, p_i32]),
    "jenga_request_release": (C.c_int, [c_vp, c_i64, c_i32]),
    "jenga_request_touch": (C.c_int, [c_vp, c_i64, c_i32, c_i64, c_i64, c_i64]),
    "jenga_request_set_prefix_lengths": (C.c_int, [c_vp, c_i64, c_i32]),
    "jenga_possible_prefixes": (C.c_int, [c_i32, c_i32, c_vp, c_i32, c_vp]),
    "jenga_longest_common_prefix": (C.c_int, [c_vp, c_i32, c_i32]),
    "jenga_kv_append": (C.c_int, [c_vp, c_i32, c_i32, c_vp, c_vp, c_vp, c_i32, c_vp, c_i32, c_vp]),
    "jenga_kv_write_range": (C.c_int, [c_vp, c_i32, c_i32, c_vp, c_vp, c_vp, c_vp, c_vp, c_i32, c_i32, c_i32, c_vp]),
    "jenga_decode_num_partitions": (C.c_int, [c_vp, c_i32, c_i32, c_i32, c_i32, c_i32, c_i32]),
    "jenga_decode_workspace_bytes": (c_i64, [c_vp, c_i32, c_i32, c_i32, c_i32, c_i32, c_i32]),
    "jenga_paged_decode": (C.c_int, [c_vp, c_i32, c_i32, c_vp, c_i32, c_vp, c_vp, c_vp, c_i32, c_vp, c_i32,
                                     c_i32, c_i32, c_f32, c_i32, c_vp, c_i64, c_vp, c_vp]),
    "jenga_paged_decode_partial": (C.c_int, [c_vp, c_i32, c_i32, c_vp, c_i32, c_vp, c_vp, c_vp, c_i32, c_vp,
                                             c_i32, c_i32, c_i32, c_f32, c_i32, c_vp, c_i64, c_vp]),
    "jenga_splitk_reduce": (C.c_int, [c_vp, c_i32, c_i32, c_vp, c_i32, c_i32, c_i32, c_i32, c_vp,
                                      c_i64, c_vp, c_vp]),
    "jenga_paged_decode_static": (C.c_int, [c_vp, c_i32, c_i32, c_vp, c_i32, c_vp, c_vp, c_vp, c_i32, c_vp, c_i32,
                                            c_i32, c_i32, c_f32, c_i32, c_vp, c_vp]),
    "jenga_stream_copy": (C.c_int, [c_vp, c_vp, c_i64, c_vp]),
    "jenga_stream_read": (C.c_int, [c_vp, c_i64, c_vp, c_vp]),
    "jenga_strerror": (C.c_char_p, [C.c_int]),
    "jenga_version": (C.c_int, []),
}

_lib = None


def load() -> C.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first "
            "(python -c 'import __graft_entry__ as g; g.build()' or python paper_2503_18292_amd/build.py)")
    lib = C.CDLL(LIB_PATH)
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)          # AttributeError if the library lacks a declared symbol
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib
