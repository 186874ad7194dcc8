"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Every case prefills the pool with NaN bytes and scatters NaN into token rows outside the
visible set, so each parity check is also a check that nothing outside the visible set is
read into the result.  Tolerances are the ones stated for this build: max abs 1e-5 for
fp32 K/V; for bf16 K/V max abs 2e-2 and relative (norm-wise) 1e-2.  Next to them stands a
regression bound at what the kernels reach with a margin: the bf16 path multiplies bf16 inputs
exactly, accumulates in fp32 and feeds the probabilities to the value product as the sum of two
bf16 numbers, so its results lie within a few 1e-6 of the oracle on unit-variance inputs; the
bound of 1e-4 (element by element) catches the loss of the second term (4e-3 on short requests,
tests/test_accuracy_model.py) or a wrong rescale, which the stated 2e-2 would let through.
"""
import math

import numpy as np
import pytest
import torch

from oracle.attn import decode_attention_one, visible_range
from workloads import configs, layout, scripts
from workloads.configs import CROSS, FULL, OPAQUE, WINDOW, KindCfg, LengthDist, ModelCfg

pytestmark = pytest.mark.gpu

TOL_F32_ABS = 1e-5
TOL_BF16_ABS = 2e-2
TOL_BF16_REL = 1e-2
REG_BF16_ABS = 1e-4       # regression bound, element-wise, for inputs of standard deviation <= 1


def _runner(cfg, seed, **kw):
    from paper_2503_18292_amd.runner import DecodeRunner
    return DecodeRunner(cfg, seed, **kw)


def prepare(r, poison=True):
    """Host step, NaN-prefilled pool, seeded contexts scattered (masked rows NaN), inputs made."""
    r.build_contexts()
    r.host_step()
    r.pool_u8.fill_(0xFF if poison else 0)
    for k, layer in r.schedule:
        kd = r.cfg.kinds[k]
        for b in range(r.cfg.batch):
            K, V = r.contiguous_kv(k, layer, b)
            L = int(r.seq_lens_host[k][b])
            n_cached = L - (0 if kd.type == CROSS else 1)
            if poison:
                lo, _ = visible_range(L, kd.window)
                K, V = K.clone(), V.clone()
                K[:, :lo] = float("nan")
                V[:, :lo] = float("nan")
            layout.scatter_request(r.pool_u8, kd, layer, r.tables_host[k][b].tolist(), K, V, n_cached)
    r.make_inputs(new_token_from_seeded_kv=True)


def check_against_oracle(r, label=""):
    torch.cuda.synchronize()
    worst = 0.0
    for k, layer in r.schedule:
        kd = r.cfg.kinds[k]
        q = r.inputs[(k, layer)][0].cpu().double().numpy()
        got = r.out[(k, layer)].cpu().double().numpy()
        for b in range(r.cfg.batch):
            K, V = r.contiguous_kv(k, layer, b)
            want = decode_attention_one(q[b], K.double().numpy(), V.double().numpy(), r.scale(k), kd.window)
            err = np.abs(got[b] - want)
            assert np.isfinite(got[b]).all(), f"{label} kind {k} layer {layer} request {b}: non-finite output"
            if kd.dtype == "f32":
                assert err.max() <= TOL_F32_ABS, f"{label} kind {k} layer {layer} req {b}: {err.max()}"
            else:
                assert err.max() <= TOL_BF16_ABS, f"{label} kind {k} layer {layer} req {b}: {err.max()}"
                rel = np.linalg.norm(got[b] - want) / max(np.linalg.norm(want), 1e-30)
                assert rel <= TOL_BF16_REL, f"{label} kind {k} layer {layer} req {b}: rel {rel}"
                reg = REG_BF16_ABS * max(1.0, r.cfg.value_sigma)
                assert err.max() <= reg, f"{label} kind {k} layer {layer} req {b}: {err.max()} above the regression bound {reg}"
            worst = max(worst, float(err.max()))
    return worst


def check_append_landed(r):
    """The appended token, read back through the harness's own address map, is bit-exact."""
    for k, layer in r.schedule:
        kd = r.cfg.kinds[k]
        if kd.type == CROSS:
            continue
        for b in range(r.cfg.batch):
            K, V = r.contiguous_kv(k, layer, b)
            Kg, Vg = r.gather(k, layer, b)
            bits = lambda t: t.contiguous().view(torch.uint8)
            assert torch.equal(bits(Kg[:, -1]), bits(K[:, -1]))
            assert torch.equal(bits(Vg[:, -1]), bits(V[:, -1]))
            lo, hi = visible_range(K.shape[1], kd.window)
            assert torch.equal(bits(Kg[:, lo:hi]), bits(K[:, lo:hi]))
            assert torch.equal(bits(Vg[:, lo:hi]), bits(V[:, lo:hi]))


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_tiny_config_exhaustive(seed):
    print(f"[case] tiny seed={seed}", flush=True)
    r = _runner(configs.tiny(), seed)
    prepare(r)
    r.device_step()
    worst = check_against_oracle(r, f"tiny/{seed}")
    check_append_landed(r)
    print(f"  worst abs err {worst:.3e}", flush=True)
    r.close()


def custom_cfg(dtype, D, Hq, Hkv, typ, window=0, batch=3, lo=1, hi=700, n_layers=2, T=16, cross_len=0):
    kind = KindCfg("k", typ, dtype, n_layers, Hq, Hkv, D, T, window=window)
    other = KindCfg("pad", OPAQUE, "f32", 1, tokens_per_page=1, opaque_page_bytes=3 * kind.slice_bytes)
    return ModelCfg(name=f"{dtype}-D{D}-G{Hq // Hkv}-{typ}", kinds=[kind, other], batch=batch,
                    ctx=LengthDist("uniform", lo, hi), cross_len=cross_len, build_chunk=64, n_dummy=1,
                    dummy_ctx=(1, 200))


SHAPES = [(dt, D, G) for dt in ("bf16", "f32") for D in (64, 128, 256) for G in (1, 2, 4, 8)]
SHAPES += [(dt, D, 16) for dt in ("bf16", "f32") for D in (64, 128, 256)]


@pytest.mark.parametrize("dtype,D,G", SHAPES)
def test_all_built_shapes_full_attention(dtype, D, G):
    print(f"[case] full {dtype} D={D} G={G}", flush=True)
    cfg = custom_cfg(dtype, D, 2 * G, 2, FULL, hi=600)
    r = _runner(cfg, 10 + D + G)
    prepare(r)
    r.device_step()
    check_against_oracle(r, cfg.name)
    check_append_landed(r)
    r.close()


@pytest.mark.parametrize("T,dtype,D,G,window", [
    (8, "bf16", 128, 2, 0), (8, "f32", 64, 4, 0), (32, "bf16", 256, 2, 0), (32, "bf16", 64, 1, 50),
    (64, "bf16", 128, 4, 0), (64, "f32", 128, 2, 70), (128, "bf16", 64, 2, 0), (128, "f32", 256, 1, 300),
    (8, "f32", 256, 2, 9)])
def test_other_page_sizes(T, dtype, D, G, window):
    """Pages of 8, 32, 64 and 128 tokens, bf16 and fp32 K/V."""
    print(f"[case] T={T} {dtype} D={D} G={G} W={window}", flush=True)
    cfg = custom_cfg(dtype, D, 2 * G, 2, WINDOW if window else FULL, window=window, hi=900, T=T)
    for pps in (0, 2):
        r = _runner(cfg, 40 + T + D, pages_per_split=pps)
        prepare(r)
        r.device_step()
        check_against_oracle(r, f"{cfg.name}/T{T}/pps{pps}")
        check_append_landed(r)
        r.close()


@pytest.mark.parametrize("T,dtype,D,G,window", [
    (1, "bf16", 128, 4, 0), (1, "f32", 64, 2, 37), (2, "bf16", 256, 2, 0), (4, "bf16", 64, 8, 0), (4, "f32", 128, 3, 21),
    (24, "bf16", 128, 4, 0), (24, "bf16", 256, 2, 100), (12, "f32", 64, 5, 0), (48, "bf16", 64, 1, 0),
    (3, "bf16", 128, 16, 50), (256, "bf16", 128, 2, 0), (20, "f32", 256, 4, 300)])
def test_any_number_of_tokens_per_page(T, dtype, D, G, window):
    """The paper leaves the page size open (Sec. 4.1 footnote: arbitrary; its figures use one token
    per page): 1, 2 and 4 tokens, and sizes that are no power of two, through the engine mode in
    which every lane looks up the page of the row it loads."""
    print(f"[case] any T={T} {dtype} D={D} G={G} W={window}", flush=True)
    # lengths up to 2500 tokens: with one token per page the page-id registers are refilled many times
    cfg = custom_cfg(dtype, D, 2 * G, 2, WINDOW if window else FULL, window=window, hi=2500 if T < 8 else 1500, T=T,
                     batch=4, n_layers=1)
    for pps in (0, 7):
        for fuse in (True, False):
            r = _runner(cfg, 90 + T + D, pages_per_split=pps, fuse_append=fuse)
            prepare(r)
            r.device_step()
            check_against_oracle(r, f"{cfg.name}/T{T}/pps{pps}")
            check_append_landed(r)
            r.close()


@pytest.mark.parametrize("D,G,window,pps,T", [
    (128, 8, 0, 0, 16), (128, 8, 200, 2, 16), (128, 16, 0, 6, 16), (64, 8, 70, 0, 16), (64, 4, 0, 4, 16),
    (256, 8, 0, 0, 16), (256, 16, 33, 1, 16), (128, 1, 0, 2, 16), (64, 16, 0, 0, 16),
    (128, 16, 100, 0, 64), (256, 2, 0, 1, 32), (64, 8, 0, 3, 128), (128, 4, 130, 0, 128), (256, 4, 0, 0, 64),
    (128, 8, 0, 0, 8), (64, 16, 21, 3, 8), (256, 2, 0, 1, 8), (128, 4, 77, 0, 8),
    (128, 3, 0, 0, 16), (128, 5, 90, 2, 16), (256, 3, 0, 0, 16), (64, 7, 0, 1, 32), (128, 6, 40, 0, 8),
    (256, 12, 0, 3, 16), (64, 15, 0, 0, 16), (128, 9, 0, 0, 64)])
def test_matrix_core_engine_shapes(D, G, window, pps, T):
    """bf16 K/V on the matrix-core engine, pages from 8 (half a 16-token block, odd page counts
    included) to 128 tokens, any number of query heads per KV head up to 16: ragged lengths from
    one token to many tiles, windows that start inside a page, partitions that cut inside a page."""
    print(f"[case] matrix-core D={D} G={G} W={window} pps={pps} T={T}", flush=True)
    cfg = custom_cfg("bf16", D, 2 * G, 2, WINDOW if window else FULL, window=window, batch=7, lo=0, hi=1300, T=T)
    r = _runner(cfg, 500 + D + G, pages_per_split=pps,
                ctx=np.array([0, 1, 15, 16, 31, 1299, 640]))
    prepare(r)
    r.device_step()
    check_against_oracle(r, cfg.name)
    check_append_landed(r)
    r.close()


@pytest.mark.parametrize("D,G,window,pps,T", [
    (64, 1, 0, 0, 16), (64, 8, 70, 2, 16), (128, 2, 0, 0, 16), (128, 8, 0, 3, 16), (128, 16, 200, 0, 16),
    (256, 2, 0, 1, 16), (256, 4, 33, 0, 16), (256, 16, 0, 0, 16), (128, 3, 0, 0, 16), (64, 7, 21, 1, 32),
    (128, 5, 0, 2, 8), (256, 1, 0, 0, 8), (64, 4, 0, 0, 128), (128, 12, 130, 0, 64), (256, 6, 0, 5, 32)])
def test_matrix_core_engine_shapes_fp32(D, G, window, pps, T):
    """fp32 K/V through the fp32 matrix-core products: the same ragged lengths, head counts 1 to 16,
    pages of 8 to 128 tokens, rows of 256 bytes to 1 KiB."""
    print(f"[case] matrix-core fp32 D={D} G={G} W={window} pps={pps} T={T}", flush=True)
    cfg = custom_cfg("f32", D, 2 * G, 2, WINDOW if window else FULL, window=window, batch=7, lo=0, hi=1300, T=T)
    r = _runner(cfg, 900 + D + G, pages_per_split=pps,
                ctx=np.array([0, 1, 15, 16, 31, 1299, 640]))
    prepare(r)
    r.device_step()
    check_against_oracle(r, cfg.name)
    check_append_landed(r)
    r.close()


@pytest.mark.parametrize("dtype,D,G,W", [("bf16", 256, 2, 100), ("bf16", 128, 4, 64), ("bf16", 64, 1, 33),
                                         ("f32", 128, 2, 32), ("f32", 64, 4, 17), ("bf16", 128, 8, 1),
                                         ("f32", 256, 1, 500), ("bf16", 256, 2, 16)])
def test_sliding_window_shapes(dtype, D, G, W):
    print(f"[case] window {dtype} D={D} G={G} W={W}", flush=True)
    cfg = custom_cfg(dtype, D, 2 * G, 2, WINDOW, window=W, hi=400)
    r = _runner(cfg, 77 + W)
    prepare(r)
    # slide-out really happened: no page wholly left of the window is resident
    for b in range(cfg.batch):
        L = int(r.seq_lens_host[0][b])
        row = r.tables_host[0][b].tolist()
        for p, sid in enumerate(row):
            touches = p * 16 < L and (p + 1) * 16 > max(0, L - W)
            assert (sid >= 0) == touches
    r.device_step()
    check_against_oracle(r, cfg.name)
    r.close()


@pytest.mark.parametrize("Lx", [1, 15, 16, 17, 404, 1601])
def test_cross_attention_ragged_encoder_length(Lx):
    print(f"[case] cross Lx={Lx}", flush=True)
    cfg = custom_cfg("bf16", 128, 8, 2, CROSS, cross_len=Lx, batch=2)
    r = _runner(cfg, 5)
    prepare(r)
    r.device_step()
    check_against_oracle(r, cfg.name)
    r.close()


@pytest.mark.parametrize("ctx", [[0, 0, 0], [15, 16, 17], [127, 128, 255], [0, 1023, 31]])
def test_edge_lengths(ctx):
    """L = 1 (a single token returns its value row), page and tile boundaries."""
    print(f"[case] edge ctx={ctx}", flush=True)
    for dtype, D in (("bf16", 256), ("f32", 64), ("bf16", 128)):
        cfg = custom_cfg(dtype, D, 4, 2, FULL)
        r = _runner(cfg, 3, ctx=np.array(ctx))
        prepare(r)
        r.device_step()
        check_against_oracle(r, cfg.name)
        for b, c in enumerate(ctx):
            if c == 0:      # one visible token: softmax weight exactly 1
                for k, layer in r.schedule:
                    V = r.contiguous_kv(k, layer, b)[1].float()
                    got = r.out[(k, layer)][b].cpu()
                    for h in range(4):
                        assert torch.equal(got[h], V[h // 2, 0])
        r.close()


def score_rounding_envelope(q, K, V, scale, window, dtype):
    """Element-wise bound [H_q, D] on |result - oracle| for arithmetic that holds each score as an
    fp32 number in the base-2 domain, derived from the oracle's own quantities in fp64.

    One rounding of a score s2 = s * log2(e) to fp32 moves it by up to ulp_fp32(s2) / 2, i.e. the
    natural score by h = ulp_fp32(s2) / 2 * ln 2.  A score goes through R such roundings: one per
    accumulator update of the dot product (D / 4 updates with fp32 operands, D / 32 with bf16
    operands, whose products are exact), the multiplication by the scale and the subtraction of
    the running maximum.  Independent roundings add in quadrature, sqrt(R) * h; the bound allows
    u = 2 * sqrt(R) * h per score.  With p = softmax(s) and out = p @ V,
    d out[d] / d s[t] = p[t] * (V[t, d] - out[d]), so every sign pattern of perturbations within
    +-u stays inside  env[d] = sum_t p[t] * |V[t, d] - out[d]| * u[t]  to first order (u < 1e-3
    here).  Added to it: the rounding of the weighted sum itself, 4 * 2^-24 * sum_t p[t] |V[t, d]|
    for an fp32 accumulation, and for bf16 K/V 2^-16 times the same sum for probabilities that
    enter the value product with 16 significant bits."""
    q, K, V = (np.asarray(x, dtype=np.float64) for x in (q, K, V))
    Hq, Hkv = q.shape[0], K.shape[0]
    G = Hq // Hkv
    R = q.shape[1] // (32 if dtype == "bf16" else 4) + 2
    lo, hi = visible_range(K.shape[1], window)
    bound = np.zeros_like(q)
    for h in range(Hq):
        Kh, Vh = K[h // G, lo:hi], V[h // G, lo:hi]
        s = scale * (Kh @ q[h])
        p = np.exp(s - s.max())
        p /= p.sum()
        out = p @ Vh
        half_ulp = np.spacing(np.abs(s * math.log2(math.e)).astype(np.float32)).astype(np.float64) / 2 * math.log(2.0)
        env = (p * 2 * math.sqrt(R) * half_ulp) @ np.abs(Vh - out)
        acc = p @ np.abs(Vh)
        bound[h] = env + (4 * 2.0 ** -24 + (2.0 ** -16 if dtype == "bf16" else 0.0)) * acc
    return bound


@pytest.mark.parametrize("dtype,D,G,T", [("bf16", 128, 4, 16), ("bf16", 256, 2, 16), ("f32", 64, 2, 16), ("bf16", 64, 8, 32),
                                         ("f32", 128, 8, 16)])
def test_peaked_softmax_large_scores(dtype, D, G, T):
    """K/V of large magnitude: scores of several hundred, the softmax is close to one-hot and the
    exponent range is only survivable through the running maximum."""
    print(f"[case] peaked {dtype} D={D} G={G} T={T}", flush=True)
    cfg = custom_cfg(dtype, D, 2 * G, 2, FULL, hi=500, T=T)
    cfg.value_sigma = 150.0
    r = _runner(cfg, 61)
    prepare(r)
    r.device_step()
    torch.cuda.synchronize()
    worst_rel = worst_ratio = 0.0
    for k, layer in r.schedule:
        kd = r.cfg.kinds[k]
        q = r.inputs[(k, layer)][0].cpu().double().numpy()
        got = r.out[(k, layer)].cpu().double().numpy()
        for b in range(cfg.batch):
            K, V = r.contiguous_kv(k, layer, b)
            want = decode_attention_one(q[b], K.double().numpy(), V.double().numpy(), r.scale(k), 0)
            assert np.isfinite(got[b]).all()
            # Outputs are of the magnitude of V here (150), and the scores of several hundred are
            # held in fp32 by any implementation of this path: the bound is what that rounding
            # allows, computed from the oracle (see score_rounding_envelope), not a constant.
            bound = score_rounding_envelope(q[b], K.double().numpy(), V.double().numpy(), r.scale(k), 0, dtype)
            excess = np.abs(got[b] - want) - bound
            assert excess.max() <= 0, f"kind {k} layer {layer} req {b}: {np.abs(got[b] - want).max()} vs bound {bound.max()}"
            ratio = float((np.abs(got[b] - want) / bound).max())
            rel = np.linalg.norm(got[b] - want) / np.linalg.norm(want)
            worst_rel, worst_ratio = max(worst_rel, rel), max(worst_ratio, ratio)
            if dtype == "bf16":
                assert rel <= TOL_BF16_REL, rel
    print(f"  worst norm-wise rel err {worst_rel:.2e}, worst error / bound {worst_ratio:.2f}", flush=True)
    r.close()


def test_empty_batch_entries_give_zeros():
    cfg = custom_cfg("bf16", 128, 4, 2, FULL)
    r = _runner(cfg, 4, ctx=np.array([40, 9, 100]))
    prepare(r)
    lens = r.seq_lens[0].clone()
    lens[1] = 0
    r.seq_lens[0] = lens
    for key in r.out:
        r.out[key].fill_(7.0)
    r.device_step()
    torch.cuda.synchronize()
    for k, layer in r.schedule:
        assert torch.equal(r.out[(k, layer)][1].cpu(), torch.zeros(4, 128))
    r.seq_lens_host[0][1] = 0
    r.close()


@pytest.mark.parametrize("dtype,D,G", [("bf16", 256, 2), ("bf16", 128, 4), ("f32", 64, 2)])
def test_split_k_choices_agree(dtype, D, G):
    """Any partition size gives the oracle's result; different sizes agree to rounding."""
    print(f"[case] split-k {dtype} D={D} G={G}", flush=True)
    outs = []
    for pps in (0, 4, 8, 64, 256):
        cfg = custom_cfg(dtype, D, 2 * G, 2, FULL, lo=900, hi=3000, n_layers=1)
        r = _runner(cfg, 21, pages_per_split=pps)
        prepare(r)
        r.device_step()
        check_against_oracle(r, f"{cfg.name}/pps{pps}")
        outs.append(r.out[(0, 0)].cpu().clone())
        r.close()
    for o in outs[1:]:
        assert (o - outs[0]).abs().max() <= (2e-6 if dtype == "f32" else 2e-5)


def test_result_does_not_depend_on_physical_placement():
    """Same tokens in different physical pages: bit-identical output."""
    cfg = custom_cfg("bf16", 256, 4, 2, FULL, lo=300, hi=900, n_layers=2)
    ctx = scripts.sample_ctx(cfg, 9)
    outs, tabs = [], []
    for script_seed in (100, 200):
        r = _runner(cfg, 9, ctx=ctx, script_seed=script_seed)
        prepare(r)
        r.device_step()
        torch.cuda.synchronize()
        outs.append({key: v.cpu().clone() for key, v in r.out.items()})
        tabs.append(r.tables_host[0].clone())
        r.close()
    assert not torch.equal(tabs[0], tabs[1]), "placements should differ"
    for key in outs[0]:
        assert torch.equal(outs[0][key], outs[1][key])


@pytest.mark.parametrize("dtype,D,G,T,window", [("bf16", 256, 2, 16, 0), ("bf16", 128, 4, 16, 70), ("f32", 64, 2, 16, 0),
                                                 ("bf16", 128, 8, 16, 0), ("bf16", 64, 2, 32, 40), ("f32", 256, 1, 16, 0)])
def test_append_inside_decode_equals_separate_append(dtype, D, G, T, window):
    """Appending inside the decode kernel gives the same pool bytes and the same outputs as
    jenga_kv_append followed by decode."""
    print(f"[case] fused append {dtype} D={D} G={G} T={T} W={window}", flush=True)
    cfg = custom_cfg(dtype, D, 2 * G, 2, WINDOW if window else FULL, window=window, hi=700, T=T, batch=5)
    ctx = scripts.sample_ctx(cfg, 61)
    ctx[0], ctx[1] = 0, 15          # a first token, and a token that fills its page
    results = []
    for fuse in (False, True):
        r = _runner(cfg, 61, ctx=ctx, fuse_append=fuse)
        prepare(r)
        r.device_step()
        check_against_oracle(r, f"{cfg.name}/fuse={fuse}")
        check_append_landed(r)
        torch.cuda.synchronize()
        results.append(({key: v.cpu().clone() for key, v in r.out.items()}, r.pool_u8.cpu().clone()))
        r.close()
    for key in results[0][0]:
        assert torch.equal(results[0][0][key], results[1][0][key])
    assert torch.equal(results[0][1], results[1][1])


def test_partial_plus_reduce_equals_fused_entry_point():
    cfg = custom_cfg("bf16", 128, 8, 2, WINDOW, window=200, lo=100, hi=1500, n_layers=1)
    r = _runner(cfg, 31, pages_per_split=4)
    prepare(r)
    r.run_layer(0, 0)
    torch.cuda.synchronize()
    fused = r.out[(0, 0)].cpu().clone()
    r.out[(0, 0)].zero_()
    r.run_layer(0, 0, split=True)
    torch.cuda.synchronize()
    assert torch.equal(fused, r.out[(0, 0)].cpu())
    r.close()


def test_opaque_pages_interleaved_and_untouched():
    """Jamba-like pool: state pages sit between KV pages and no kernel writes them."""
    cfg = configs.jamba_like()
    cfg.batch = 6
    for kd in cfg.kinds:
        if kd.type == OPAQUE:     # smaller state pages keep the test pool small; ratios stay uneven
            kd.n_layers, kd.opaque_page_bytes = 1, 7 * cfg.kinds[0].small_page_bytes
    cfg.ctx = LengthDist("lognormal", 128, 2000, median=400.0, sigma=1.0)
    cfg.build_chunk = 64
    r = _runner(cfg, 2)
    prepare(r)
    sentinel = 0x5A
    state_ids = [r.pool.request_block_table_row(req, 1, 1)[0] for req in r.requests]
    S = cfg.kinds[1].small_page_bytes
    for sid in state_ids:
        r.pool_u8[sid * S:(sid + 1) * S] = sentinel
    owners = [r.pool.large_page_owner(i)[0] for i in range(r.n_large)]
    used = [o for o in owners if o >= 0]
    assert any(a != b for a, b in zip(used, used[1:])), "kinds should interleave in the pool"
    r.device_step()
    check_against_oracle(r, "jamba-small")
    for sid in state_ids:
        assert bool((r.pool_u8[sid * S:(sid + 1) * S] == sentinel).all())
    r.close()


def test_prefix_sharing_reads_shared_pages():
    cfg = configs.long_5to1()
    cfg.batch = 8
    cfg.share_tokens, cfg.share_fraction = 256, 0.5
    cfg.ctx = LengthDist("uniform", 256, 1500)
    for kd in cfg.kinds:
        kd.n_layers = 1
        kd.window = 128 if kd.type == WINDOW else 0
    cfg.build_chunk = 128
    r = _runner(cfg, 12)
    r.build_contexts()
    r.host_step()
    group = scripts.sharers(cfg, r.ctx, 12)
    assert len(group) >= 2
    # sharers hold the same physical pages for the shared prefix of the full kind
    lead_row = r.tables_host[1][group[0]][:16]
    for b in group[1:]:
        assert torch.equal(r.tables_host[1][b][:16], lead_row)
    # values: the sharers' first 256 tokens must be the leader's, since the pages are the same
    orig = r.contiguous_kv

    def shared_kv(k, layer, b):
        K, V = orig(k, layer, b)
        if k == 1 and b in group[1:]:
            Kl, Vl = orig(k, layer, group[0])
            K, V = K.clone(), V.clone()
            K[:, :256], V[:, :256] = Kl[:, :256], Vl[:, :256]
        return K, V

    r.contiguous_kv = shared_kv
    r._built = True
    r.pool_u8.fill_(0xFF)
    for k, layer in r.schedule:
        kd = cfg.kinds[k]
        for b in range(cfg.batch):
            K, V = r.contiguous_kv(k, layer, b)
            layout.scatter_request(r.pool_u8, kd, layer, r.tables_host[k][b].tolist(), K, V,
                                   int(r.seq_lens_host[k][b]) - 1)
    r.make_inputs(new_token_from_seeded_kv=True)
    r.device_step()
    check_against_oracle(r, "prefix-sharing")
    r.close()


def test_bad_table_entries_are_clamped_not_followed():
    """Entries of the visible range that are negative or past the pool are a caller error; the
    kernels clamp them (reads) or skip them (writes), so other requests are unaffected."""
    cfg = custom_cfg("bf16", 128, 8, 2, FULL, lo=100, hi=600, n_layers=1, batch=4)
    for fuse in (True, False):
        r = _runner(cfg, 17, fuse_append=fuse)
        prepare(r)
        before = r.pool_u8.clone()
        tab = r.tables[0].clone()
        tab[1, :] = -1
        tab[2, 0] = 2 ** 30
        tab[2, int(r.seq_lens_host[0][2] - 1) // 16] = 2 ** 30      # the page the append would write
        r.tables[0] = tab
        r.device_step()
        torch.cuda.synchronize()
        got = r.out[(0, 0)].cpu().double().numpy()
        q = r.inputs[(0, 0)][0].cpu().double().numpy()
        for b in (0, 3):
            K, V = r.contiguous_kv(0, 0, b)
            want = decode_attention_one(q[b], K.double().numpy(), V.double().numpy(), r.scale(0), 0)
            assert np.abs(got[b] - want).max() <= REG_BF16_ABS
        # nothing was written for the two requests with bad tables: only requests 0 and 3 appended
        changed = (r.pool_u8 != before).sum().item()
        assert changed <= 2 * 2 * 2 * 128 * 2
        r.close()


def test_device_entry_points_reject_bad_arguments():
    import paper_2503_18292_amd as J
    cfg = custom_cfg("bf16", 128, 4, 2, FULL)
    r = _runner(cfg, 1)
    prepare(r)
    q, k_new, v_new = r.inputs[(0, 0)]
    with pytest.raises(J.JengaError) as e:      # workspace too small
        r.pool.paged_decode(0, 0, q, r.tables[0], r.seq_lens[0], r.max_len[0], 0, 0.1,
                            r.workspace[0][:4], r.out[(0, 0)])
    assert e.value.status == -4
    with pytest.raises(J.JengaError):           # block table narrower than max_seq_len
        r.pool.paged_decode(0, 0, q, r.tables[0][:, :1].contiguous(), r.seq_lens[0], 4096, 0, 0.1,
                            r.workspace[0], r.out[(0, 0)])
    with pytest.raises(J.JengaError):           # layer out of range
        r.pool.kv_append(0, 99, k_new, v_new, r.tables[0], r.seq_lens[0])
    with pytest.raises(J.JengaError):           # OPAQUE kind has no kernels
        r.pool.kv_append(1, 0, k_new, v_new, r.tables[0], r.seq_lens[0])
    with pytest.raises(J.JengaError) as e:      # misaligned q
        base = torch.empty(q.numel() + 8, dtype=q.dtype, device=q.device)
        q_mis = base[1:1 + q.numel()].view(q.shape)          # 2 bytes off a 16-byte boundary
        r.pool.paged_decode(0, 0, q_mis, r.tables[0], r.seq_lens[0], r.max_len[0],
                            0, 0.1, r.workspace[0], r.out[(0, 0)])
    assert e.value.status == -3
    torch.cuda.synchronize()
    r.close()
