"""jenga_paged_decode_static (the entry point that allocates nothing) against jenga_paged_decode.

The static variant keeps its split-K records in the library's own device buffer; everything else
is shared with the ordinary entry point, so the outputs must be bit-identical.  Two calls in a
row, the second with a smaller input, so that stale records of the first call lie in the buffer
when the second runs.  Collected last: it must pass alone in a fresh process and after the
other tests.
"""
import numpy as np
import pytest
import torch

from workloads.configs import FULL, WINDOW

from test_gpu_parity import _runner, check_against_oracle, custom_cfg, prepare

pytestmark = pytest.mark.gpu


def _both(r, k, layer, lens, batch, fused, window=None):
    """(workspace entry point, static entry point) outputs for the first `batch` requests."""
    kd = r.cfg.kinds[k]
    window = kd.window if window is None else window
    q, k_new, v_new = r.inputs[(k, layer)]
    kn, vn = (k_new[:batch], v_new[:batch]) if fused else (None, None)
    a = torch.full((batch, kd.n_q_heads, kd.head_dim), 3.0, dtype=torch.float32, device="cuda")
    b = torch.full_like(a, 5.0)
    r.pool.paged_decode(k, layer, q[:batch], r.tables[k][:batch], lens[:batch], r.max_len[k], window,
                        r.scale(k), r.workspace[k], a, 0, kn, vn)
    r.pool.paged_decode_static(k, layer, q[:batch], r.tables[k][:batch], lens[:batch], r.max_len[k], window,
                               r.scale(k), b, 0, kn, vn)
    torch.cuda.synchronize()
    return a.cpu(), b.cpu()


@pytest.mark.parametrize("dtype,D,G,window,batch", [("bf16", 128, 4, 0, 40), ("bf16", 256, 2, 300, 9), ("f32", 64, 2, 0, 17)])
def test_static_scratch_entry_point_matches_the_workspace_one(dtype, D, G, window, batch):
    print(f"[case] static scratch {dtype} D={D} G={G} W={window} batch={batch}", flush=True)
    cfg = custom_cfg(dtype, D, 2 * G, 2, WINDOW if window else FULL, window=window, batch=batch, lo=1, hi=2500,
                     n_layers=1)
    r = _runner(cfg, 31 + batch)
    prepare(r)
    k, layer = r.schedule[0]
    # first call: the whole batch, append fused (both entry points store the same rows)
    a, b = _both(r, k, layer, r.seq_lens[k], batch, fused=True)
    assert torch.equal(a, b)
    r.out[(k, layer)].copy_(b.cuda())
    check_against_oracle(r, cfg.name)                      # and the oracle agrees, to the usual bar
    # second call right after it, stale records of the first in the buffer: fewer requests, and
    # fewer visible tokens each (half the length; a sliding-window kind keeps only its window's
    # pages resident, so there the window is narrowed instead)
    small = max(1, batch // 3)
    if window:
        a2, b2 = _both(r, k, layer, r.seq_lens[k], small, fused=False, window=window // 3)
    else:
        a2, b2 = _both(r, k, layer, torch.clamp(r.seq_lens[k] // 2, min=1), small, fused=False)
    assert bool(torch.isfinite(a2).all())
    assert torch.equal(a2, b2)
    assert not torch.equal(a2, a[:small])                  # really another result
    r.close()


def test_static_scratch_limit_is_reported():
    """More records than the 32 MiB buffer holds: a clear error, nothing launched."""
    import paper_2503_18292_amd as J
    cfg = custom_cfg("bf16", 256, 128, 8, FULL, batch=2, n_layers=1)        # G = 16, 256-element heads
    r = _runner(cfg, 3)
    prepare(r)
    B = 1024
    q = torch.zeros(B, 128, 256, dtype=torch.bfloat16, device="cuda")
    table = torch.zeros(B, r.tables[0].shape[1], dtype=torch.int32, device="cuda")
    lens = torch.ones(B, dtype=torch.int32, device="cuda")
    out = torch.empty(B, 128, 256, dtype=torch.float32, device="cuda")
    with pytest.raises(J.JengaError) as e:
        r.pool.paged_decode_static(0, 0, q, table, lens, r.max_len[0], 0, 0.1, out)
    assert e.value.status == -4          # JENGA_ERR_WORKSPACE
    torch.cuda.synchronize()
    r.close()


def test_static_entry_point_in_a_hip_graph():
    """What the entry point is for: captured into a HIP graph (where nothing may be allocated) and
    replayed, with eager work and synchronisations between the replays, it gives the result of the
    eager workspace call every time, append included."""
    cfg = custom_cfg("bf16", 128, 8, 2, FULL, batch=6, lo=300, hi=3000, n_layers=2)
    r = _runner(cfg, 91)
    prepare(r)
    r.device_step()                                        # eager, workspace entry point, append fused
    torch.cuda.synchronize()
    check_against_oracle(r, "eager")
    eager = {key: v.clone() for key, v in r.out.items()}
    pool_after = r.pool_u8.clone()

    def static_step():
        for k, layer in r.schedule:
            kd = r.cfg.kinds[k]
            q, k_new, v_new = r.inputs[(k, layer)]
            r.pool.paged_decode_static(k, layer, q, r.tables[k], r.seq_lens[k], r.max_len[k], kd.window,
                                       r.scale(k), r.out[(k, layer)], 0, k_new, v_new)

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            static_step()
    torch.cuda.current_stream().wait_stream(side)
    other = torch.zeros(1 << 20, device=r.device)
    for rep in range(3):
        for v in r.out.values():
            v.fill_(float("nan"))
        other.add_(1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for key in eager:
            assert torch.equal(r.out[key], eager[key]), f"replay {rep} layer {key}"
        assert torch.equal(r.pool_u8, pool_after)          # the appended rows are the same rows
    r.close()
