"""A whole decode step recorded into a HIP graph and replayed gives the eager result every time.

The library's device entry points allocate nothing, synchronise nothing and record no memset,
so a caller may capture them.  The graph is replayed several times with the program's own eager
work and synchronisations between the replays, and every replay is checked."""
import numpy as np
import pytest
import torch

from workloads.configs import FULL, WINDOW

from test_gpu_parity import _runner, check_against_oracle, custom_cfg, prepare

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,D,G,typ,window", [("bf16", 256, 2, FULL, 0), ("bf16", 128, 4, WINDOW, 90)])
def test_decode_step_in_a_hip_graph(dtype, D, G, typ, window):
    cfg = custom_cfg(dtype, D, 2 * G, 2, typ, window=window, lo=200, hi=900, n_layers=3, batch=4)
    r = _runner(cfg, 33)
    prepare(r)
    r.device_step()                      # eager: also lets the library cache its launch geometry
    check_against_oracle(r, "eager")
    eager = {key: v.clone() for key, v in r.out.items()}
    pool_after = r.pool_u8.clone()

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            r.device_step()
    torch.cuda.current_stream().wait_stream(side)
    scratch = torch.zeros(1 << 20, device=r.device)
    for rep in range(4):
        for v in r.out.values():
            v.fill_(float("nan"))
        scratch.add_(1.0)                # unrelated eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for key in eager:
            assert torch.equal(r.out[key], eager[key]), f"replay {rep} layer {key}"
        assert torch.equal(r.pool_u8, pool_after)
    check_against_oracle(r, "graph")
    r.close()


def test_decode_step_on_a_side_stream():
    """The kernels run on the stream they are given: a step issued on a non-default stream while
    the default stream is kept busy gives the eager result."""
    cfg = custom_cfg("bf16", 128, 8, 2, FULL, lo=100, hi=1200, n_layers=2, batch=5)
    r = _runner(cfg, 44)
    prepare(r)
    r.device_step()
    torch.cuda.synchronize()
    eager = {key: v.clone() for key, v in r.out.items()}
    for v in r.out.values():
        v.fill_(float("nan"))
    side = torch.cuda.Stream()
    busy = torch.zeros(1 << 26, device=r.device)
    side.wait_stream(torch.cuda.current_stream())
    for _ in range(20):
        busy.add_(1.0)                   # the default stream has its own work meanwhile
    with torch.cuda.stream(side):
        r.device_step()
    side.synchronize()
    for key in eager:
        assert torch.equal(r.out[key], eager[key]), key
    torch.cuda.synchronize()
    r.close()
