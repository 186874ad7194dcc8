"""GPU parity at the limits of what the kernels accept: the largest batch whose prefix sums every
block makes for itself, batches beyond it (prefix sums from a kernel of their own), one very long
request next to very short ones, and lengths above the stated maximum (clamped by the kernels)."""
import numpy as np
import pytest
import torch

from workloads.configs import FULL, WINDOW

from test_gpu_parity import _runner, check_against_oracle, check_append_landed, custom_cfg, prepare

pytestmark = pytest.mark.gpu

MAX_BATCH = 1024      # the largest batch whose prefix sums are made per block, in LDS


@pytest.mark.parametrize("batch,T,dtype,D,G,window", [
    (MAX_BATCH, 16, "bf16", 128, 4, 0),      # matrix-core engine
    (MAX_BATCH, 32, "f32", 64, 2, 40),       # fp32 K/V, 32-token pages, sliding window
    (65, 16, "bf16", 256, 2, 0),             # 512-byte rows, one page per tile; one request past a full round of the length scan
    (200, 16, "f32", 64, 1, 0),
    (256, 16, "bf16", 128, 4, 0),            # the last batch of the four-round form of the length scan
    (257, 8, "bf16", 64, 4, 0),              # the first of the sixteen-round form, 8-token pages
    (777, 16, "f32", 128, 2, 30),            # a ragged last round
])
def test_large_batches(batch, T, dtype, D, G, window):
    print(f"[case] batch={batch} T={T} {dtype} D={D} G={G} W={window}", flush=True)
    typ = WINDOW if window else FULL
    cfg = custom_cfg(dtype, D, 2 * G, 2, typ, window=window, batch=batch, lo=0, hi=90, n_layers=1, T=T)
    r = _runner(cfg, 77 + batch)
    prepare(r)
    r.device_step()
    check_against_oracle(r, cfg.name)
    check_append_landed(r)
    r.close()


@pytest.mark.parametrize("dtype,window", [("bf16", 0), ("f32", 50)])
def test_many_segments_per_wavefront_append_runs_in_front(dtype, window):
    """Batch 1024 with 8 KV heads: 8192 (request, KV head) segments for 1024 wavefronts, where the
    library runs the append as a launch of its own in front of the decode kernel although the new
    rows were passed to the decode call.  Outputs and pool contents must be what the fused path gives."""
    print(f"[case] many segments {dtype} W={window}", flush=True)
    cfg = custom_cfg(dtype, 64, 16, 8, WINDOW if window else FULL, window=window, batch=MAX_BATCH, lo=0, hi=70,
                     n_layers=1)
    r = _runner(cfg, 4242)
    prepare(r)
    r.device_step()
    check_against_oracle(r, cfg.name)
    check_append_landed(r)
    r.close()


@pytest.mark.parametrize("batch,T,dtype,D,G,window,hi", [
    (MAX_BATCH + 1, 16, "bf16", 128, 4, 0, 60),      # one request past the per-block scan
    (4096, 16, "bf16", 128, 4, 0, 90),               # the case the larger decode batches of the paper point to
    (3000, 32, "f32", 64, 2, 50, 120),               # fp32 K/V, sliding window, 32-token pages
    (5000, 8, "bf16", 64, 3, 0, 40),                 # 8-token pages, run-time head count, three rounds of the search
])
def test_batches_beyond_the_per_block_scan(batch, T, dtype, D, G, window, hi):
    print(f"[case] big batch={batch} T={T} {dtype} D={D} G={G} W={window}", flush=True)
    typ = WINDOW if window else FULL
    cfg = custom_cfg(dtype, D, 2 * G, 2, typ, window=window, batch=batch, lo=0, hi=hi, n_layers=1, T=T)
    r = _runner(cfg, 7 + batch)
    prepare(r)
    r.device_step()
    check_against_oracle(r, cfg.name)
    check_append_landed(r)
    r.close()


def test_batch_above_the_grid_limit_is_refused():
    import paper_2503_18292_amd as J
    cfg = custom_cfg("bf16", 128, 4, 2, FULL, batch=2, n_layers=1)
    r = _runner(cfg, 1)
    with pytest.raises(J.JengaError) as e:
        r.pool.decode_workspace_bytes(0, 4, 65536, 64)
    assert e.value.status == -6      # JENGA_ERR_UNSUPPORTED
    assert r.pool.decode_workspace_bytes(0, 4, 65535, 64) > 0
    r.close()


@pytest.mark.parametrize("dtype,D,G,window", [("bf16", 128, 4, 0), ("bf16", 256, 2, 0), ("bf16", 128, 4, 1024)])
def test_one_very_long_request_among_short_ones(dtype, D, G, window):
    """131072 tokens (the longest length of the synthetic workloads) next to 1- and 6-token
    requests: almost every wavefront works on the long request, a few segments are tiny."""
    print(f"[case] long request {dtype} D={D} G={G} W={window}", flush=True)
    typ = WINDOW if window else FULL
    cfg = custom_cfg(dtype, D, 2 * G, 2, typ, window=window, batch=3, n_layers=1)
    r = _runner(cfg, 9, ctx=np.array([0, 131071, 5]))
    prepare(r)
    r.device_step()
    check_against_oracle(r, cfg.name)
    check_append_landed(r)
    r.close()


@pytest.mark.parametrize("T,D,G,pps", [(8, 128, 4, 0), (8, 64, 16, 700), (128, 256, 2, 0), (32, 128, 8, 300),
                                         (16, 128, 4, 1000), (16, 256, 2, 500), (16, 64, 8, 4000)])
def test_long_request_other_page_sizes(T, D, G, pps):
    """Thousands of pages per request; with large partitions one wavefront walks through many runs
    of 64 pages, so its page-id registers are refilled again and again."""
    print(f"[case] long request T={T} D={D} G={G} pps={pps}", flush=True)
    cfg = custom_cfg("bf16", D, 2 * G, 2, FULL, batch=3, n_layers=1, T=T)
    r = _runner(cfg, 19, ctx=np.array([30001, 7, 12345]), pages_per_split=pps)
    prepare(r)
    r.device_step()
    check_against_oracle(r, cfg.name)
    check_append_landed(r)
    r.close()


def test_lengths_above_max_seq_len_are_clamped():
    """A length above max_seq_len is treated as max_seq_len: the result is that of the clamped
    length, and nothing past the table's width is read."""
    cfg = custom_cfg("bf16", 128, 4, 2, FULL, n_layers=1)
    ctx = np.array([100, 37, 63])
    r = _runner(cfg, 2, ctx=ctx)
    prepare(r)
    k, layer = r.schedule[0]
    q = r.inputs[(k, layer)][0]
    cap = 64                                           # a page boundary below two of the lengths
    lens_clamped = torch.minimum(r.seq_lens[k], torch.tensor(cap, dtype=torch.int32, device="cuda"))
    want = torch.empty_like(r.out[(k, layer)])
    got = torch.empty_like(want)
    table = r.tables[k][:, :cap // 16].contiguous()
    r.pool.kv_append(k, layer, *r.inputs[(k, layer)][1:], r.tables[k], r.seq_lens[k])
    r.pool.paged_decode(k, layer, q, table, lens_clamped, cap, 0, r.scale(k), r.workspace[k], want)
    r.pool.paged_decode(k, layer, q, table, r.seq_lens[k], cap, 0, r.scale(k), r.workspace[k], got)
    torch.cuda.synchronize()
    assert torch.equal(got.cpu(), want.cpu())
    # the same with the new rows handed to the decode call: a request whose length exceeds
    # max_seq_len is attended as clamped and its rows are NOT stored (row max_seq_len - 1 holds a
    # valid cached token); requests within the bound are appended as usual
    k_new, v_new = r.inputs[(k, layer)][1:]
    before = r.pool_u8.clone()
    got2 = torch.empty_like(want)
    r.pool.paged_decode(k, layer, q, table, r.seq_lens[k], cap, 0, r.scale(k), r.workspace[k], got2, 0, k_new, v_new)
    torch.cuda.synchronize()
    assert torch.equal(got2.cpu(), want.cpu())        # the row of request 1 was already in the pool: same bytes
    assert torch.equal(r.pool_u8.cpu(), before.cpu())
    # max_seq_len = 0 with positive lengths: nothing visible, zeros out, nothing read or stored
    got3 = torch.full_like(want, 7.0)
    r.pool.paged_decode(k, layer, q, table, r.seq_lens[k], 0, 0, r.scale(k), r.workspace[k], got3, 0, k_new, v_new)
    torch.cuda.synchronize()
    assert float(got3.abs().max()) == 0.0 and torch.equal(r.pool_u8.cpu(), before.cpu())
    r.close()


def test_clamped_request_is_not_appended_when_the_append_runs_in_front():
    """Batch 1024 x 8 KV heads (the library runs the append as its own launch in front): a request
    longer than max_seq_len is skipped by that launch exactly as by the fused path."""
    cfg = custom_cfg("bf16", 64, 16, 8, FULL, batch=MAX_BATCH, lo=0, hi=40, n_layers=1)
    r = _runner(cfg, 5)
    prepare(r)
    k, layer = r.schedule[0]
    q, k_new, v_new = r.inputs[(k, layer)]
    lens = r.seq_lens[k].clone()
    cap = r.max_len[k]
    over = [3, 500, 1023]
    lens[over] = cap + 5                              # caller error: beyond what the launch was sized for
    before = r.pool_u8.clone()
    out = torch.empty_like(r.out[(k, layer)])
    r.pool.paged_decode(k, layer, q, r.tables[k], lens, cap, 0, r.scale(k), r.workspace[k], out, 0, k_new, v_new)
    torch.cuda.synchronize()
    # expected pool: the separate append with the clamped requests left out
    lens_ok = r.seq_lens[k].clone()
    lens_ok[over] = 0
    after = r.pool_u8.clone()
    r.pool_u8.copy_(before)
    r.pool.kv_append(k, layer, k_new, v_new, r.tables[k], lens_ok)
    torch.cuda.synchronize()
    assert torch.equal(after.cpu(), r.pool_u8.cpu())
    # the other requests are served as ever (the partition boundaries moved, so not bit for bit)
    ref = torch.empty_like(out)
    r.pool.paged_decode(k, layer, q, r.tables[k], r.seq_lens[k], cap, 0, r.scale(k), r.workspace[k], ref)
    torch.cuda.synchronize()
    keep = torch.ones(MAX_BATCH, dtype=torch.bool)
    keep[over] = False
    assert torch.allclose(out.cpu()[keep], ref.cpu()[keep], atol=1e-4, rtol=0)
    r.close()
