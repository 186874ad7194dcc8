"""The prefix-cache side of the allocator (Sec. 5) together with the kernels.

Request 1 is served and finishes with its pages kept as cache.  Request 2 shares its first
tokens: it takes the cached pages back into use (a prefix hit), gets pages of its own for the
rest, and decodes through a block table that mixes both -- the result must be the oracle's on
the joined history.  Then request 3 needs more pages than are free: the five-step allocation
evicts what is left of request 1's cache, the eviction reports name exactly those pages, none of
them is in a live block table, and request 2 still decodes to the same result afterwards.
"""
import numpy as np
import pytest
import torch

from oracle.attn import decode_attention_one
from workloads import layout, values
from workloads.configs import FULL, KindCfg

import paper_2503_18292_amd as J
from paper_2503_18292_amd import api
from paper_2503_18292_amd.api import make_kind

from test_gpu_parity import REG_BF16_ABS

pytestmark = pytest.mark.gpu


def decode_one(pool, kd, layer, q, row, L, width):
    table = torch.full((1, width), -1, dtype=torch.int32)
    table[0, :len(row)] = torch.tensor(row, dtype=torch.int32)
    table_d = table.cuda()
    lens = torch.tensor([L], dtype=torch.int32, device="cuda")
    ws = torch.empty(pool.decode_workspace_bytes(0, kd.n_q_heads, 1, width * kd.tokens_per_page) // 4,
                     dtype=torch.float32, device="cuda")
    out = torch.empty(1, kd.n_q_heads, kd.head_dim, dtype=torch.float32, device="cuda")
    pool.paged_decode(0, layer, q, table_d, lens, width * kd.tokens_per_page, 0, kd.head_dim ** -0.5, ws, out)
    torch.cuda.synchronize()
    return out[0].cpu().double().numpy()


@pytest.mark.parametrize("T,r_large", [(16, 1), (16, 4), (8, 2)])
def test_prefix_hit_then_eviction_under_pressure(T, r_large):
    print(f"[case] prefix cache T={T} small pages per large page={r_large}", flush=True)
    kd = KindCfg("full", FULL, "bf16", 2, 8, 2, 128, T)
    S = kd.small_page_bytes
    n_large = 24 // r_large * 2                       # 48 small pages
    mem = torch.full((n_large * r_large * S,), 0xFF, dtype=torch.uint8, device="cuda")
    pool = J.Pool(mem.data_ptr(), mem.numel(), [make_kind(J.FULL, J.BF16, 2, 2, 128, T)], large_page_bytes=r_large * S)
    width = 48
    layer = 1

    # ---- request 1: 20 pages of history, served, finished, kept as cache
    L1 = 20 * T
    K1, V1 = values.kv_for_request(kd, layer, 1, L1, 1.0, 5)
    pool.request_extend(1, 0, L1)
    row1 = pool.request_block_table_row(1, 0, 20)
    layout.scatter_request(mem, kd, layer, row1, K1, V1, L1)
    pool.request_touch(1, 0, 0, L1, 10)               # update_last_access: full attention stamps everything
    pool.request_set_prefix_lengths(1, 0)
    pool.request_release(1, keep_cached=True)
    assert pool.kind_stats(0).evictable_small_pages == 20 and pool.kind_stats(0).used_small_pages == 0

    # ---- request 2: shares the first 12 pages (a prefix hit), 5 pages of its own, then one decode step
    hit_pages = 12
    for sid in row1[:hit_pages]:
        pool.acquire_cached(0, sid)
        pool.set_last_access(0, sid, 20)
    L2 = (hit_pages + 5) * T - 3                      # the last page is partly filled
    own, evicted = [], []
    for _ in range(5):
        sid, ev = pool.alloc_small_evict(0, 2)
        own.append(sid)
        evicted += ev
    assert evicted == []                              # 48 - 20 pages were still empty
    row2 = row1[:hit_pages] + own
    K2, V2 = values.kv_for_request(kd, layer, 2, L2, 1.0, 5)
    K2[:, :hit_pages * T], V2[:, :hit_pages * T] = K1[:, :hit_pages * T], V1[:, :hit_pages * T]   # the shared history
    # only request 2's own tokens are written: the shared ones are already in the cached pages
    own_row = [-1] * hit_pages + own
    layout.scatter_request(mem, kd, layer, own_row, K2, V2, L2)
    q = values.normal((1, kd.n_q_heads, kd.head_dim), "bf16", 1.0, 5, 77).cuda()
    got = decode_one(pool, kd, layer, q, row2, L2, width)
    want = decode_attention_one(q[0].cpu().double().numpy(), K2.double().numpy(), V2.double().numpy(), kd.head_dim ** -0.5, 0)
    assert np.abs(got - want).max() <= REG_BF16_ABS

    # ---- request 3: needs more than the empty pages: what is left of request 1's cache is evicted
    row3, reports = [], []
    n_empty = 48 - 20 - 5
    for i in range(n_empty + 6):
        sid, ev = pool.alloc_small_evict(0, 3)
        row3.append(sid)
        reports += ev
    gone = {sid for _, sid in reports}
    assert len(reports) == len(gone) >= 6 and all(k == 0 for k, _ in reports)
    assert gone <= set(row1[hit_pages:])              # only unused cache, never a page request 2 uses
    # evicted pages are request 3's now (or empty again, in a large page that became request 3's)
    # and appear in no other live table
    assert not (gone & set(row2)) and len(gone & set(row3)) >= 6
    for sid in gone:
        assert pool.small_state(0, sid) != api.PAGE_EVICTABLE
    assert len(set(row3)) == len(row3) and not (set(row3) & set(row2))
    for sid in row2 + row3:
        assert pool.small_state(0, sid) == api.PAGE_USED
    # request 3 writes its pages; request 2 still reads its own history
    K3, V3 = values.kv_for_request(kd, layer, 3, len(row3) * T, 1.0, 5)
    layout.scatter_request(mem, kd, layer, row3, K3, V3, len(row3) * T)
    again = decode_one(pool, kd, layer, q, row2, L2, width)
    assert np.array_equal(again, got)
    got3 = decode_one(pool, kd, layer, q, row3, len(row3) * T, width)
    want3 = decode_attention_one(q[0].cpu().double().numpy(), K3.double().numpy(), V3.double().numpy(), kd.head_dim ** -0.5, 0)
    assert np.abs(got3 - want3).max() <= REG_BF16_ABS
    # everything released without caching: the pool drains
    for sid in row2 + row3:
        pool.release_small(0, sid, keep_cached=False)
    for sid in set(row1[hit_pages:]) - gone:
        pool.acquire_cached(0, sid)
        pool.free_small(0, sid)
    info = pool.get_info()
    assert info.free_large_pages == info.n_large_pages
    pool.destroy()
