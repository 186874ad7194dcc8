"""GPU parity on seeded random cases: shape, page size, window, partition size, batch and
lengths all drawn from the seed, each case checked element by element against the oracle and
for the appended token.  Catches combinations the hand-picked cases do not list."""
import numpy as np
import pytest

from workloads.configs import FULL, WINDOW

from test_gpu_parity import _runner, check_against_oracle, check_append_landed, custom_cfg, prepare

pytestmark = pytest.mark.gpu


def draw_case(seed):
    rng = np.random.default_rng(1000 + seed)
    dtype = rng.choice(["bf16", "bf16", "f32"])
    D = int(rng.choice([64, 128, 256]))
    T = int(rng.choice([16, 16, 16, 8, 32, 64, 128, 1, 4, 24, 10]))
    G = int(rng.choice([1, 2, 4, 8, 16, 3, 5, 6, 7, 12]))
    Hkv = int(rng.choice([1, 2, 3]))
    window = int(rng.choice([0, 0, rng.integers(1, 400)]))
    # partitions of 150 and 1000 pages make one wavefront walk through several runs of 64 pages
    pps = int(rng.choice([0, 0, 1, 2, 3, 5, 8, 40, 150, 1000]))
    batch = int(rng.integers(1, 9))
    hi = int(rng.choice([40, 300, 1200, 6000]))     # up to 750 pages of 8 tokens: several refills of the page-id registers
    ctx = rng.integers(0, hi, size=batch)
    # lengths that sit on page and tile boundaries are the interesting ones: plant a few
    for i in range(batch):
        if rng.random() < 0.3:
            ctx[i] = max(0, int(rng.choice([T, 2 * T, 4 * T, 64, 128])) * int(rng.integers(1, 5)) - int(rng.integers(0, 3)))
    return dtype, D, T, G, Hkv, window, pps, ctx


@pytest.mark.parametrize("seed", range(64))
def test_random_case(seed):
    dtype, D, T, G, Hkv, window, pps, ctx = draw_case(seed)
    print(f"[case] random {seed}: {dtype} D={D} T={T} G={G} Hkv={Hkv} W={window} pps={pps} ctx={ctx.tolist()}", flush=True)
    cfg = custom_cfg(dtype, D, G * Hkv, Hkv, WINDOW if window else FULL, window=window, batch=len(ctx),
                     n_layers=int(1 + seed % 2), T=T)
    r = _runner(cfg, 2000 + seed, pages_per_split=pps, ctx=ctx)
    prepare(r)
    r.device_step()
    check_against_oracle(r, f"random/{seed}")
    check_append_landed(r)
    r.close()
