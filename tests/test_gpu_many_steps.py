"""GPU parity over a run of decode steps: block tables change from step to step (new pages at
page boundaries, sliding-window pages freed), every step appends one token per request through
the decode call, and at every step the outputs are checked against the oracle on the history the
test keeps itself, and the pool -- read back through the harness's own address map -- against that
history bit for bit."""
import numpy as np
import pytest
import torch

from oracle.attn import decode_attention_one, visible_range
from workloads.configs import FULL, WINDOW
from workloads import values

from test_gpu_parity import (REG_BF16_ABS, TOL_BF16_ABS, TOL_BF16_REL, TOL_F32_ABS, _runner, check_against_oracle,
                             check_append_landed, custom_cfg, prepare)

pytestmark = pytest.mark.gpu

STEPS = 40


@pytest.mark.parametrize("dtype,D,G,window,T,fuse", [
    ("bf16", 128, 4, 0, 16, True), ("bf16", 128, 4, 40, 16, True), ("bf16", 256, 2, 25, 8, True),
    ("f32", 64, 2, 33, 32, True), ("bf16", 64, 8, 0, 16, False)])
def test_appends_accumulate_over_many_steps(dtype, D, G, window, T, fuse):
    print(f"[case] {STEPS} steps {dtype} D={D} G={G} W={window} T={T} fuse={fuse}", flush=True)
    cfg = custom_cfg(dtype, D, 2 * G, 2, WINDOW if window else FULL, window=window, batch=3, T=T, n_layers=2)
    # contexts next to page boundaries, so that the run crosses several of them
    r = _runner(cfg, 5, ctx=np.array([T - 2, 2 * T - 1, 3 * T]), fuse_append=fuse, step_budget=STEPS + 2)
    prepare(r)
    r.device_step()
    check_against_oracle(r, "step 0")
    check_append_landed(r)
    hist = {}
    for k, layer in r.schedule:
        for b in range(cfg.batch):
            hist[(k, layer, b)] = r.contiguous_kv(k, layer, b)          # [H_kv, L, D], storage dtype, CPU
    tdt = values.TORCH_DTYPE[dtype]
    gen = torch.Generator().manual_seed(1234)
    bits = lambda t: t.contiguous().view(torch.uint8)
    for step in range(1, STEPS + 1):
        r.advance()                                  # one token longer: allocator calls, new tables on the device
        for k, layer in r.schedule:
            kd = cfg.kinds[k]
            q, _, _ = r.inputs[(k, layer)]
            k_new = (torch.randn(cfg.batch, kd.n_kv_heads, kd.head_dim, generator=gen) * 0.7).to(tdt)
            v_new = (torch.randn(cfg.batch, kd.n_kv_heads, kd.head_dim, generator=gen) * 0.7).to(tdt)
            r.inputs[(k, layer)] = (q, k_new.to(r.device), v_new.to(r.device))
            for b in range(cfg.batch):
                K, V = hist[(k, layer, b)]
                hist[(k, layer, b)] = (torch.cat([K, k_new[b][:, None, :]], dim=1),
                                       torch.cat([V, v_new[b][:, None, :]], dim=1))
        r.device_step()
        torch.cuda.synchronize()
        for k, layer in r.schedule:
            kd = cfg.kinds[k]
            q = r.inputs[(k, layer)][0].cpu().double().numpy()
            got = r.out[(k, layer)].cpu().double().numpy()
            for b in range(cfg.batch):
                K, V = hist[(k, layer, b)]
                L = K.shape[1]
                assert L == int(r.seq_lens_host[k][b])
                want = decode_attention_one(q[b], K.double().numpy(), V.double().numpy(), r.scale(k), kd.window)
                err = np.abs(got[b] - want).max()
                assert np.isfinite(got[b]).all()
                if dtype == "f32":
                    assert err <= TOL_F32_ABS, (step, k, layer, b, err)
                else:
                    rel = np.linalg.norm(got[b] - want) / max(np.linalg.norm(want), 1e-30)
                    assert err <= TOL_BF16_ABS and rel <= TOL_BF16_REL, (step, k, layer, b, err, rel)
                    assert err <= REG_BF16_ABS, (step, k, layer, b, err)      # regression bound (test_gpu_parity)
                Kg, Vg = r.gather(k, layer, b)
                lo, hi = visible_range(L, kd.window)
                assert torch.equal(bits(Kg[:, lo:hi]), bits(K[:, lo:hi])), (step, k, layer, b)
                assert torch.equal(bits(Vg[:, lo:hi]), bits(V[:, lo:hi])), (step, k, layer, b)
    r.close()
