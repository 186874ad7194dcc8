#!/usr/bin/env python3
"""Benchmark: decode steps of a synthetic heterogeneous-KV workload on one MI355X.

A step is the whole hot path once: the host allocator makes room for every request's
new token (two-level LCM pool, request-aware placement, window slide-out), block tables
and lengths go to the device, and for each attention layer in model order the new K/V is
appended and paged decode attention (partial + split-K reduce) runs through that layer
type's block table.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line: metric = K/V bytes read per second over whole steps, plus
`roofline` for the dominant kernel (timed with events on the launch stream inside the
timed region) and `cpu_baseline` (the CPU oracle timed on a bounded sample).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E peak
# HBM traffic of one decode_partial launch.  NOT measured in this run (counters need the
# profiler): derived from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this same program, each
# counter scaled by what it reads for a plain copy of known size (summaries and commands:
# profiles/decode_kernels_*_hbm_traffic.md).  roofline.traffic = fetch_over_algorithmic x the
# run's algorithmic bytes per launch + write_bytes; roofline.traffic_source says so.
MEASURED_TRAFFIC = {"gemma2_9b": {"fetch_over_algorithmic": 1.004, "write_bytes": 3.69e6},
                    "llama32_vision_11b": {"fetch_over_algorithmic": 1.0075, "write_bytes": 2.60e6},
                    "jamba_like": {"fetch_over_algorithmic": 1.0043, "write_bytes": 4.75e6},
                    "long_5to1": {"fetch_over_algorithmic": 1.0047, "write_bytes": 2.55e6},
                    "short_b1024": {"fetch_over_algorithmic": 1.025, "write_bytes": 1.871e7}}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gemma2_9b",
                    choices=["tiny", "gemma2_9b", "llama32_vision_11b", "jamba_like", "long_5to1",
                             "short_b1024", "jamba_like_literal"])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--pages-per-split", type=int, default=0, help="0: library's choice")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="do not bracket the decode kernel with events (roofline.achieved becomes null)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=30.0,
                    help="wall-clock budget of the CPU-oracle leg (reading slices back, converting, oracle)")
    ap.add_argument("--mode", default="decode", choices=["decode", "kv_write", "allocator"],
                    help="decode: the benchmark proper; kv_write: bulk K/V write of a prefill chunk; "
                         "allocator: host microseconds per allocator call, library against oracle")
    ap.add_argument("--chunk", type=int, default=512, help="kv_write: tokens written per request and call")
    ap.add_argument("--hip-graph", action="store_true",
                    help="record the device side of a step (all layers) into a HIP graph once and replay "
                         "it in the timed region; the host step and table copies stay eager")
    ap.add_argument("--copy-calibration", type=float, default=0.0, metavar="GiB",
                    help="instead of the benchmark, run the library's plain copy and read kernels over "
                         "a buffer of this size (to calibrate profiler byte counters) and exit")
    return ap.parse_args()


def host_info():
    """What the CPU figures ran on: cores this process may use, and the CPU's name."""
    try:
        affinity = len(os.sched_getaffinity(0))
    except AttributeError:
        affinity = os.cpu_count() or 1
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for ln in f:
                if ln.lower().startswith("model name"):
                    model = ln.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return affinity, model


def cpu_baseline(runner, budget_s: float, fast_budget_s: float = 8.0):
    """The fp64 oracle on the host cores, on (request, layer) slices gathered from the pool.
    `budget_s` bounds the wall-clock time of the whole leg (most of it goes into reading the
    slices back and converting them to fp64); only the oracle's own time enters the rate.
    `cores` is the number of cores the oracle kept busy (its CPU time over its wall-clock time,
    rounded): its per-head matrix-vector products leave most BLAS threads idle.
    A second figure, clearly labelled, comes from oracle/attn_threads.py (fp32, one task per
    (request, KV head) on a thread pool) on slices of the same step, so that the CPU side of the
    report is not only a deliberately plain loop."""
    import numpy as np
    import torch
    from oracle.attn import decode_attention_one
    from oracle.attn_threads import decode_attention_threads
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threadpool_limits = None
        blas_threads = 1
    affinity, cpu_model = host_info()
    torch.cuda.synchronize()
    t_used, cpu_used, nbytes, n_units = 0.0, 0.0, 0, 0
    leg_t0 = time.perf_counter()
    per_kind = {}
    for ki, k in enumerate(runner.attn_kinds):
        kd = runner.cfg.kinds[k]
        t_kind, b_kind, n_kind = 0.0, 0, 0
        share = budget_s * (ki + 1) / len(runner.attn_kinds)
        for layer in range(kd.n_layers):
            q = runner.inputs[(k, layer)][0].cpu().double().numpy()
            for b in range(runner.cfg.batch):
                if time.perf_counter() - leg_t0 >= share:
                    break
                K, V = runner.gather(k, layer, b)
                Kd, Vd = K.double().numpy(), V.double().numpy()
                vis = int(runner.visible_tokens(k)[b])
                Kd[:, :Kd.shape[1] - vis] = 0.0      # rows outside the window are never read by the oracle
                Vd[:, :Vd.shape[1] - vis] = 0.0
                t0, c0 = time.perf_counter(), time.process_time()
                decode_attention_one(q[b], Kd, Vd, runner.scale(k), kd.window)
                dt = time.perf_counter() - t0
                cpu_used += time.process_time() - c0
                t_used += dt
                t_kind += dt
                b_kind += vis * kd.bytes_per_token_per_layer
                n_kind += 1
            if time.perf_counter() - leg_t0 >= share:
                break
        per_kind[k] = (t_kind, b_kind, n_kind)
        nbytes += b_kind
        n_units += n_kind
    gbs = nbytes / t_used / 1e9 if t_used > 0 else 0.0
    # scale the sample to a whole step: every layer of a kind has the same shapes
    step_s = 0.0
    for k, (t_kind, b_kind, n_kind) in per_kind.items():
        if b_kind:
            step_s += t_kind * runner.kv_bytes_layer(k) / b_kind * runner.cfg.kinds[k].n_layers
    out = {
        "value": round(gbs, 4), "unit": "GB/s", "cores": max(1, int(round(cpu_used / t_used))) if t_used > 0 else 1,
        "kind": "oracle",
        "cores_note": "cores = CPU time / wall-clock time inside the oracle (what it kept busy)",
        "host": {"cores_available": affinity, "cpu_model": cpu_model, "blas_threads": blas_threads},
        "sample": f"{n_units} (request, layer) slices of the same step, read back from the pool: layers then "
                  f"requests in order, each attention kind until its share of {budget_s:.0f} s of wall-clock "
                  f"time (read-back and conversion included) is used; fp64 numpy, {t_used:.1f} s inside the oracle; "
                  f"scaled to a whole step by bytes and "
                  f"layer count: {step_s:.1f} s/step = {runner.cfg.batch / step_s if step_s else 0:.3f} tokens/s",
        "seconds": round(t_used, 2),
    }
    # second figure: fp32, one task per (request, KV head) on all available cores; batches of
    # requests of layer 0 of each kind until the budget is used
    fast_t, fast_bytes, fast_n = 0.0, 0, 0
    fast_t0 = time.perf_counter()
    threads = max(1, affinity)
    limit = threadpool_limits(limits=1) if threadpool_limits else None    # the pool's threads are the parallelism
    try:
        for k in runner.attn_kinds:
            kd = runner.cfg.kinds[k]
            q32 = runner.inputs[(k, 0)][0].cpu().float().numpy()
            b0 = 0
            while b0 < runner.cfg.batch and time.perf_counter() - fast_t0 < fast_budget_s:
                bs = list(range(b0, min(runner.cfg.batch, b0 + 2 * threads)))
                Ks, Vs = [], []
                for b in bs:
                    K, V = runner.gather(k, 0, b)
                    Ks.append(K.float().numpy())
                    Vs.append(V.float().numpy())
                t0 = time.perf_counter()
                decode_attention_threads(q32[bs], Ks, Vs, runner.scale(k), kd.window, threads)
                fast_t += time.perf_counter() - t0
                fast_bytes += sum(int(runner.visible_tokens(k)[b]) for b in bs) * kd.bytes_per_token_per_layer
                fast_n += len(bs)
                b0 += len(bs)
    finally:
        if limit is not None:
            limit.restore_original_limits() if hasattr(limit, "restore_original_limits") else limit.unregister()
    out["fp32_threaded"] = {
        "value": round(fast_bytes / fast_t / 1e9, 3) if fast_t > 0 else 0.0, "unit": "GB/s", "cores": threads,
        "kind": "oracle/attn_threads.py: fp32, one task per (request, KV head) on a thread pool (not the parity oracle)",
        "sample": f"{fast_n} (request, layer 0) slices of the same step within {fast_budget_s:.0f} s of wall-clock time "
                  f"(read-back and conversion included, {fast_t:.2f} s inside the computation)",
    }
    return out


def stream_read_rate(pool_u8, nbytes: int = 8 << 30, reps: int = 5) -> float:
    """GB/s of the library's plain non-temporal read stream over the first bytes of the pool:
    the rate the memory system gives a kernel that does nothing but read."""
    import torch
    import paper_2503_18292_amd as J
    n = min(nbytes, pool_u8.numel()) // 4096 * 4096
    if n == 0:
        return 0.0
    sink = torch.zeros(4, dtype=torch.int32, device=pool_u8.device)
    J.stream_read(pool_u8, n, sink)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        J.stream_read(pool_u8, n, sink)
    e1.record()
    torch.cuda.synchronize()
    return n * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def copy_calibration(gib: float):
    """Known traffic for counter calibration: copy reads N and writes N bytes, read reads N."""
    import torch
    import paper_2503_18292_amd as J
    n = int(gib * 2**30) // 4096 * 4096
    src = torch.empty(n, dtype=torch.uint8, device="cuda")
    src.fill_(1)
    dst = torch.empty_like(src)
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    out = {"bytes": n}
    for name, fn, moved in (("copy", lambda: J.stream_copy(dst, src, n), 2 * n),
                            ("read", lambda: J.stream_read(src, n, sink), n)):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[name + "_GBps"] = round(moved / (e0.elapsed_time(e1) / 5 * 1e-3) / 1e9, 1)
    print(json.dumps({"copy_calibration": out}), flush=True)


def kv_write_bench(args):
    """Bulk K/V write (jenga_kv_write_range): every request writes its last `chunk` cached tokens."""
    import numpy as np
    import torch
    from paper_2503_18292_amd.runner import DecodeRunner
    from workloads import configs, values
    cfg = configs.ALL[args.workload]()
    r = DecodeRunner(cfg, args.seed)
    r.build_contexts()
    r.host_step()
    dev = r.device
    out = {}
    for k in r.attn_kinds:
        kd = cfg.kinds[k]
        if kd.type == configs.CROSS:
            continue
        B = cfg.batch
        n = np.minimum(args.chunk, r.ctx).astype(np.int32)
        cu = np.zeros(B + 1, dtype=np.int32)
        cu[1:] = np.cumsum(n)
        total = int(cu[-1])
        # several distinct sources in rotation, so a call never finds its input in the 256 MB
        # memory-side cache left there by the previous call
        one = values.normal((2, total, kd.n_kv_heads, kd.head_dim), kd.dtype, cfg.value_sigma, args.seed, 9).to(dev)
        srcs = [one] + [one.clone() for _ in range(5)]
        cu_d = torch.from_numpy(cu).to(dev)
        start = torch.from_numpy((r.ctx - n).astype(np.int32)).to(dev)
        layers = list(range(kd.n_layers))
        for layer in layers[:2]:
            r.pool.kv_write_range(k, layer, one[0], one[1], cu_d, start, r.tables[k])
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            for layer in layers:
                src = srcs[layer % len(srcs)]
                r.pool.kv_write_range(k, layer, src[0], src[1], cu_d, start, r.tables[k])
        e1.record()
        torch.cuda.synchronize()
        nbytes = total * kd.bytes_per_token_per_layer
        us = e0.elapsed_time(e1) * 1e3 / (args.steps * len(layers))
        # every byte is read once from the source and written once into the pool
        out[kd.name] = {"tokens_per_call": total, "bytes_written_per_call": nbytes, "us_per_call": round(us, 2),
                        "write_GBps": round(nbytes / us / 1e3, 1), "read_plus_write_GBps": round(2 * nbytes / us / 1e3, 1)}
    print(json.dumps({"mode": "kv_write", "workload": cfg.name, "chunk": args.chunk, "kinds": out,
                      "roofline": {"bound": "hbm", "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                   "achieved": max(v["read_plus_write_GBps"] for v in out.values()),
                                   "frac": round(max(v["read_plus_write_GBps"] for v in out.values()) / HBM_PEAK_GBS, 4)}}),
          flush=True)
    r.close()


def allocator_bench(args):
    """Host cost of the allocator: the workload's build + step + finish scripts, library and oracle."""
    from oracle.alloc import OraclePool, OracleRequests, lcm_bytes
    from paper_2503_18292_amd import api
    from paper_2503_18292_amd.runner import kind_descs
    from workloads import configs, scripts
    cfg = configs.ALL[args.workload]()
    ctx = scripts.sample_ctx(cfg, args.seed)
    ops = (scripts.build_script(cfg, ctx, args.seed) + scripts.step_script(cfg, ctx)
           + scripts.finish_script(cfg, args.seed))
    descs = kind_descs(cfg)
    large = api.lcm_page_bytes(descs)
    n_large = cfg.pool_large_pages or scripts.pool_large_pages_needed(cfg, ctx, large)
    lib = api.Pool(None, n_large * large, descs)
    t0 = time.perf_counter()
    scripts.run_script(ops, lib)
    t_lib = time.perf_counter() - t0
    pages = sum(-(-int(c + 1) // k.tokens_per_page) for c in ctx for k in cfg.kinds if k.type in ("full", "window"))
    S = [k.small_page_bytes for k in cfg.kinds]
    ora_pool = OraclePool(n_large * lcm_bytes(S), S)
    ora = OracleRequests(ora_pool, [k.tokens_per_page for k in cfg.kinds], [k.window for k in cfg.kinds])
    t0 = time.perf_counter()
    scripts.run_script(ops, ora)
    t_ora = time.perf_counter() - t0
    print(json.dumps({"mode": "allocator", "workload": cfg.name, "script_ops": len(ops),
                      "small_pages_allocated_at_least": pages,
                      "library_seconds": round(t_lib, 4), "library_us_per_page": round(t_lib / pages * 1e6, 3),
                      "oracle_seconds": round(t_ora, 3), "oracle_us_per_page": round(t_ora / pages * 1e6, 2),
                      "note": "library time includes the ctypes call per request-level op"}), flush=True)


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2503_18292_amd import _lib
    from paper_2503_18292_amd.runner import DecodeRunner
    from workloads import configs

    _lib.load()     # no library, no benchmark: there is no other path
    if args.copy_calibration > 0:
        return copy_calibration(args.copy_calibration)
    if args.mode == "allocator":
        return allocator_bench(args)
    if args.mode == "kv_write":
        return kv_write_bench(args)
    cfg = configs.ALL[args.workload]()
    total_steps = 2 * args.steps + args.warmup
    t_setup = time.perf_counter()
    r = DecodeRunner(cfg, args.seed, pages_per_split=args.pages_per_split, step_budget=total_steps + 2)
    r.build_contexts()
    r.host_step()
    r.fill_pool_random()
    r.make_inputs(new_token_from_seeded_kv=False)
    torch.cuda.synchronize()
    print(f"[bench] {cfg.name}: pool {r.pool_u8.numel() / 2**30:.1f} GiB in {r.n_large} large pages of "
          f"{r.large_bytes // 1024} KiB; batch {cfg.batch}; ctx {int(r.ctx.min())}..{int(r.ctx.max())}; "
          f"setup {time.perf_counter() - t_setup:.1f} s", file=sys.stderr, flush=True)

    def one_step(events=None):
        r.advance()
        r.device_step(events)

    # step 0 of the runner was the host_step above; run its device part as the first warmup
    r.device_step()
    for _ in range(max(0, args.warmup - 1)):
        one_step()
    torch.cuda.synchronize()

    graph = None
    if args.hip_graph:
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                r.device_step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()

        def one_step(events=None):           # noqa: F811  (replaces the eager step)
            r.advance()
            if events is None:
                graph.replay()
            else:
                r.device_step(events)

    # Timed region: exactly `steps` whole steps between two synchronisations -> value.
    step_bytes = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step()
        step_bytes.append(r.kv_bytes_step())
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    elapsed = t1 - t0
    ms_per_step = elapsed / args.steps * 1e3
    total_bytes = float(sum(step_bytes))
    gbs = total_bytes / elapsed / 1e9
    tokens_per_s = cfg.batch * args.steps / elapsed

    # The same number of steps again, now with a pair of events around every launch of the
    # dominant kernel (on the stream it is launched on).  Kept out of the region above because
    # each event record costs a few microseconds between kernels, 84 times per step.
    use_events = not args.no_kernel_events
    ev, layer_bytes = [], []
    ms_per_step_events = None
    if use_events:
        for _ in range(args.steps):
            ev.append({key: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                       for key in r.schedule})
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for i in range(args.steps):
            one_step(ev[i])
            layer_bytes.append({k: r.kv_bytes_layer(k) for k in r.attn_kinds})
        torch.cuda.synchronize()
        ms_per_step_events = (time.perf_counter() - t2) / args.steps * 1e3

    # what a plain read stream gets from the same memory, measured after the timed regions
    stream_gbs = stream_read_rate(r.pool_u8) if use_events else 0.0
    roof = {"bound": "hbm", "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": None,
            "traffic": None, "kernel": "decode_partial_kernel"}
    if use_events:
        k_ms, k_bytes, n_launch = 0.0, 0.0, 0
        per_kind_ms = {k: 0.0 for k in r.attn_kinds}
        per_kind_bytes = {k: 0.0 for k in r.attn_kinds}
        launch_ms = []
        for i in range(args.steps):
            for (k, layer), (e0, e1) in ev[i].items():
                ms = e0.elapsed_time(e1)
                launch_ms.append(ms)
                k_ms += ms
                k_bytes += layer_bytes[i][k]
                per_kind_ms[k] += ms
                per_kind_bytes[k] += layer_bytes[i][k]
                n_launch += 1
        achieved = k_bytes / (k_ms * 1e-3) / 1e9
        roof.update({
            "achieved": round(achieved, 1), "frac": round(achieved / HBM_PEAK_GBS, 4),
            "launches": n_launch, "avg_launch_us": round(k_ms / n_launch * 1e3, 2),
            "median_launch_us": round(float(np.median(launch_ms)) * 1e3, 2),
            "min_launch_us": round(min(launch_ms) * 1e3, 2),
            "ms_per_step_with_events": round(ms_per_step_events, 3),
            "stream_read_GBps": round(stream_gbs, 1),
            "frac_of_stream_read": round(achieved / stream_gbs, 4) if stream_gbs > 0 else None,
            "algorithmic_bytes_per_launch": round(k_bytes / n_launch),
            "traffic": (round(MEASURED_TRAFFIC[cfg.name]["fetch_over_algorithmic"] * k_bytes / n_launch
                              + MEASURED_TRAFFIC[cfg.name]["write_bytes"])
                        if cfg.name in MEASURED_TRAFFIC and args.pages_per_split == 0 else None),
            "traffic_source": (f"profiles/decode_kernels_{cfg.name}_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE, "
                               f"WRITE_SIZE, copy-calibrated): fetched = "
                               f"{MEASURED_TRAFFIC[cfg.name]['fetch_over_algorithmic']} x algorithmic, "
                               f"written = {MEASURED_TRAFFIC[cfg.name]['write_bytes']:.3g} B per launch"
                               if cfg.name in MEASURED_TRAFFIC and args.pages_per_split == 0 else None),
            "per_kind_GBps": {cfg.kinds[k].name: round(per_kind_bytes[k] / (per_kind_ms[k] * 1e-3) / 1e9, 1)
                              for k in r.attn_kinds},
        })

    line = {
        "metric": "paged-decode KV read GB/s (% HBM peak) and decode tokens/s, 1 MI355X",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.kinds[r.attn_kinds[0]].dtype,
        "data": "synthetic",
        "config": {"workload": cfg.name, "batch": cfg.batch, "kv_storage": cfg.kinds[r.attn_kinds[0]].dtype,
                   "accumulate": "f32",
                   "ctx_tokens": [int(r.ctx.min()), int(r.ctx.max())],
                   "attention_layers": len(r.schedule), "kv_bytes_per_step": int(step_bytes[-1]),
                   "pool_GiB": round(r.pool_u8.numel() / 2**30, 1)},
        "tokens_per_s": round(tokens_per_s, 1),
        "hip_graph": bool(args.hip_graph),
        "pct_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(r, args.cpu_seconds)
    print(json.dumps(line), flush=True)
    r.close()


if __name__ == "__main__":
    main()
