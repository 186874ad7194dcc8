"""Bulk K/V write (chunked prefill) through the C ABI: bit-exact placement, then decode parity.

The check of placement is the harness's own address map (workloads/layout.py), written
independently of the library; the check of the values' use is the attention oracle.
"""
import numpy as np
import pytest
import torch

from oracle.attn import visible_range
from workloads.configs import CROSS, FULL, WINDOW

from test_gpu_parity import _runner, check_against_oracle, check_append_landed, custom_cfg

pytestmark = pytest.mark.gpu


def write_contexts_through_library(r, n_chunks=2, pad_rows=3):
    """Every cached token of every (kind, layer, request), in n_chunks calls per layer."""
    dev = r.device
    B = r.cfg.batch
    for k, layer in r.schedule:
        kd = r.cfg.kinds[k]
        kv = [r.contiguous_kv(k, layer, b) for b in range(B)]
        cached = [int(r.seq_lens_host[k][b]) - (0 if kd.type == CROSS else 1) for b in range(B)]
        for ch in range(n_chunks):
            lo = [cached[b] * ch // n_chunks for b in range(B)]
            hi = [cached[b] * (ch + 1) // n_chunks for b in range(B)]
            cu = np.zeros(B + 1, dtype=np.int32)
            cu[1:] = np.cumsum([h - l for l, h in zip(lo, hi)])
            total = int(cu[-1]) + pad_rows
            k_src = torch.zeros(total, kd.n_kv_heads, kd.head_dim, dtype=kv[0][0].dtype)
            v_src = torch.zeros_like(k_src)
            for b in range(B):
                k_src[cu[b]:cu[b + 1]] = kv[b][0][:, lo[b]:hi[b]].transpose(0, 1)
                v_src[cu[b]:cu[b + 1]] = kv[b][1][:, lo[b]:hi[b]].transpose(0, 1)
            r.pool.kv_write_range(k, layer, k_src.to(dev), v_src.to(dev), torch.from_numpy(cu).to(dev),
                                  torch.tensor(lo, dtype=torch.int32, device=dev), r.tables[k])
    torch.cuda.synchronize()


@pytest.mark.parametrize("dtype,D,G,typ,window,T", [
    ("bf16", 256, 2, FULL, 0, 16), ("bf16", 128, 4, WINDOW, 100, 16), ("f32", 64, 2, FULL, 0, 16),
    ("bf16", 128, 4, CROSS, 0, 16), ("f32", 128, 1, WINDOW, 33, 16), ("bf16", 128, 8, FULL, 0, 64),
    ("bf16", 64, 16, WINDOW, 150, 32), ("f32", 256, 2, FULL, 0, 8), ("bf16", 128, 4, FULL, 0, 1),
    ("bf16", 128, 2, WINDOW, 70, 24), ("f32", 64, 4, CROSS, 0, 5)])
def test_write_range_then_decode(dtype, D, G, typ, window, T):
    print(f"[case] write_range {dtype} D={D} G={G} {typ} W={window} T={T}", flush=True)
    cfg = custom_cfg(dtype, D, 2 * G, 2, typ, window=window, hi=500, cross_len=333, batch=4, T=T)
    r = _runner(cfg, 8)
    r.build_contexts()
    r.host_step()
    r.pool_u8.fill_(0xFF)
    r.make_inputs(new_token_from_seeded_kv=True)
    write_contexts_through_library(r)
    # placement: every visible cached token reads back bit-exactly through the harness's map
    for k, layer in r.schedule:
        kd = cfg.kinds[k]
        for b in range(cfg.batch):
            K, V = r.contiguous_kv(k, layer, b)
            Kg, Vg = r.gather(k, layer, b)
            L = K.shape[1]
            lo, hi = visible_range(L, kd.window)
            hi_cached = hi - (0 if kd.type == CROSS else 1)
            bits = lambda t: t.contiguous().view(torch.uint8)
            assert torch.equal(bits(Kg[:, lo:hi_cached]), bits(K[:, lo:hi_cached]))
            assert torch.equal(bits(Vg[:, lo:hi_cached]), bits(V[:, lo:hi_cached]))
    r.device_step()
    check_against_oracle(r, cfg.name)
    check_append_landed(r)
    r.close()


def test_write_range_skips_non_resident_pages_and_padding():
    cfg = custom_cfg("bf16", 128, 4, 2, WINDOW, window=40, lo=200, hi=400, batch=3)
    r = _runner(cfg, 9)
    r.build_contexts()
    r.host_step()
    r.pool_u8.fill_(0x11)
    before = r.pool_u8.clone()
    r.make_inputs(new_token_from_seeded_kv=True)
    write_contexts_through_library(r, n_chunks=1, pad_rows=5)
    changed = (r.pool_u8 != before)
    # only bytes inside resident pages of the window kind may have changed
    S = cfg.kinds[0].small_page_bytes
    resident = torch.zeros(r.pool_u8.numel(), dtype=torch.bool, device=r.device)
    for b in range(cfg.batch):
        for sid in r.tables_host[0][b].tolist():
            if sid >= 0:
                resident[sid * S:(sid + 1) * S] = True
    assert not bool((changed & ~resident).any())
    assert bool(changed.any())
    r.close()
