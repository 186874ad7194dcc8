"""Drives one decode step of a synthetic workload through the library on one GPU.

Plumbing only: device memory comes from torch, every allocator decision and every
kernel comes from libjenga.so through the binding.  Used by the GPU tests, the smoke
check and the benchmark.  Never imports the oracle.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Tuple

import numpy as np
import torch

from workloads import configs, layout, scripts, values
from workloads.configs import CROSS, FULL, OPAQUE, WINDOW, ModelCfg

from . import api
from .api import Pool, make_kind

_TYPE = {FULL: api.FULL, WINDOW: api.WINDOW, CROSS: api.CROSS, OPAQUE: api.OPAQUE}
_DTYPE = {"f32": api.F32, "bf16": api.BF16}


def kind_descs(cfg: ModelCfg):
    out = []
    for k in cfg.kinds:
        if k.type == OPAQUE:
            out.append(make_kind(api.OPAQUE, _DTYPE[k.dtype], k.n_layers, 0, 0, 1, 0, k.small_page_bytes))
        else:
            out.append(make_kind(_TYPE[k.type], _DTYPE[k.dtype], k.n_layers, k.n_kv_heads, k.head_dim,
                                 k.tokens_per_page, k.window, 0))
    return out


class DecodeRunner:
    """Pool + block tables + per-layer inputs of one decode step of `cfg`."""

    def __init__(self, cfg: ModelCfg, seed: int, device: str = "cuda:0",
                 ctx: Optional[np.ndarray] = None, pages_per_split: int = 0,
                 script_seed: Optional[int] = None, step_budget: int = 0,
                 pool_u8: Optional[torch.Tensor] = None, fuse_append: bool = True):
        if not torch.cuda.is_available():
            raise RuntimeError("DecodeRunner needs a GPU")
        self.cfg, self.seed, self.device = cfg, seed, torch.device(device)
        self.pages_per_split = pages_per_split
        self.fuse_append = fuse_append            # append inside the decode kernel, or as its own launch
        self.script_seed = seed if script_seed is None else script_seed   # placement only
        self.ctx = scripts.sample_ctx(cfg, seed) if ctx is None else np.asarray(ctx, dtype=np.int64)
        self.descs = kind_descs(cfg)
        self.large_bytes = api.lcm_page_bytes(self.descs)
        n_large = cfg.pool_large_pages
        if n_large is None:       # room for the contexts and for the decode steps still to come
            n_large = scripts.pool_large_pages_needed(cfg, self.ctx + step_budget, self.large_bytes)
        self.n_large = n_large
        if pool_u8 is None:
            pool_u8 = torch.empty(n_large * self.large_bytes, dtype=torch.uint8, device=self.device)
        assert pool_u8.numel() >= n_large * self.large_bytes      # device memory may be handed in
        self.pool_u8 = pool_u8
        assert self.pool_u8.data_ptr() % 256 == 0
        self.pool = Pool(self.pool_u8.data_ptr(), self.pool_u8.numel(), self.descs)
        self.requests = [scripts.request_id(b) for b in range(cfg.batch)]
        self.schedule = configs.layer_schedule(cfg)
        self.attn_kinds = sorted({k for k, _ in self.schedule})
        self._built = False
        self.step_budget = step_budget           # further decode steps the tables must have room for
        self._step_no = 0
        self._pinned: Dict[int, list] = {}
        self.tables: Dict[int, torch.Tensor] = {}
        self.tables_host: Dict[int, torch.Tensor] = {}
        self.seq_lens: Dict[int, torch.Tensor] = {}
        self.seq_lens_host: Dict[int, np.ndarray] = {}
        self.max_len: Dict[int, int] = {}
        self.workspace: Dict[int, torch.Tensor] = {}
        self.out: Dict[Tuple[int, int], torch.Tensor] = {}
        self.inputs: Dict[Tuple[int, int], Tuple[torch.Tensor, Optional[torch.Tensor], Optional[torch.Tensor]]] = {}

    # ---- host side of the step -----------------------------------------------
    def build_contexts(self) -> None:
        """Allocator work that brings every request to ctx[b] cached tokens."""
        scripts.run_script(scripts.build_script(self.cfg, self.ctx, self.script_seed), self.pool)
        self._built = True

    def host_step(self) -> None:
        """Host side of one decode step: room for the new token of every request (one
        allocator call per kind and request, new pages only when a page boundary is crossed;
        window kinds drop pages that slid out), then block tables and lengths to the device."""
        assert self._built
        B = self.cfg.batch
        req_arr = np.asarray(self.requests, dtype=np.int64)
        new_len = np.ascontiguousarray(self.ctx + 1, dtype=np.int64)
        first = not self.tables
        for k in self.attn_kinds:
            kd = self.cfg.kinds[k]
            if kd.type == CROSS:
                if not first:
                    continue                      # encoder K/V never changes after the first step
                lens = np.full(B, self.cfg.cross_len, dtype=np.int32)
            else:
                self.pool.requests_extend(k, req_arr, new_len)
                lens = new_len.astype(np.int32)
            self.seq_lens_host[k] = lens
            if first:
                cap = int(lens.max()) + (0 if kd.type == CROSS else self.step_budget)
                self.max_len[k] = cap
                width = -(-cap // kd.tokens_per_page)
                self._pinned[k] = [(torch.empty(B, width, dtype=torch.int32).pin_memory(),
                                    torch.empty(B, dtype=torch.int32).pin_memory(), None)
                                   for _ in range(2)]
                self.tables[k] = torch.empty(B, width, dtype=torch.int32, device=self.device)
                self.seq_lens[k] = torch.empty(B, dtype=torch.int32, device=self.device)
                ws = self.pool.decode_workspace_bytes(k, kd.n_q_heads, B, cap, kd.window,
                                                      self.pages_per_split)
                self.workspace[k] = torch.empty(ws // 4, dtype=torch.float32, device=self.device)
            assert int(lens.max()) <= self.max_len[k], "step budget exhausted"
            slot = self._step_no % 2
            tab, ln, ev = self._pinned[k][slot]
            if ev is not None:
                ev.synchronize()                  # the copy that last used this staging buffer is done
            self.pool.block_table_fill(k, req_arr, tab)
            ln.copy_(torch.from_numpy(lens))
            self.tables[k].copy_(tab, non_blocking=True)
            self.seq_lens[k].copy_(ln, non_blocking=True)
            ev = torch.cuda.Event()
            ev.record()
            self._pinned[k][slot] = (tab, ln, ev)
            self.tables_host[k] = tab
        self._step_no += 1

    def advance(self) -> None:
        """The next decode step: every request is one token longer."""
        self.ctx = self.ctx + 1
        self.host_step()

    # ---- data -------------------------------------------------------------------
    def fill_pool_random(self) -> None:
        """Every element of the pool ~ N(0, sigma) in the attention dtype (chunked, on the GPU)."""
        dts = {self.cfg.kinds[k].dtype for k in self.attn_kinds}
        assert len(dts) == 1
        dt = values.TORCH_DTYPE[dts.pop()]
        typed = self.pool_u8.view(dt)
        gen = torch.Generator(device=self.device)
        gen.manual_seed(self.seed * 7919 + 1)
        chunk = 1 << 28
        for begin in range(0, typed.numel(), chunk):
            n = min(chunk, typed.numel() - begin)
            x = torch.randn(n, generator=gen, device=self.device, dtype=torch.float32)
            typed[begin:begin + n] = (x * self.cfg.value_sigma).to(dt)
            del x

    def contiguous_kv(self, k: int, layer: int, b: int):
        """Seeded contiguous K, V [H_kv, L_b, D] of request b in (kind k, layer), CPU."""
        kd = self.cfg.kinds[k]
        L = int(self.seq_lens_host[k][b])
        return values.kv_for_request(kd, layer, self.requests[b] * 131 + k, L,
                                     self.cfg.value_sigma, self.seed)

    def scatter_seeded_contexts(self) -> None:
        """Small configs: write the seeded K/V of all cached tokens (not the new one) into the pool."""
        for k, layer in self.schedule:
            kd = self.cfg.kinds[k]
            for b in range(self.cfg.batch):
                K, V = self.contiguous_kv(k, layer, b)
                n_cached = int(self.seq_lens_host[k][b]) - (0 if kd.type == CROSS else 1)
                layout.scatter_request(self.pool_u8, kd, layer, self.tables_host[k][b].tolist(), K, V,
                                       n_cached)

    def make_inputs(self, new_token_from_seeded_kv: bool) -> None:
        """q (and k_new, v_new for self-attention kinds) of every scheduled layer, on the device."""
        B = self.cfg.batch
        for k, layer in self.schedule:
            kd = self.cfg.kinds[k]
            q = values.q_for_layer(kd, layer * 16 + k, B, 1.0, self.seed).to(self.device)
            k_new = v_new = None
            if kd.type != CROSS:
                if new_token_from_seeded_kv:
                    rows = [self.contiguous_kv(k, layer, b) for b in range(B)]
                    k_new = torch.stack([r[0][:, -1, :] for r in rows]).contiguous().to(self.device)
                    v_new = torch.stack([r[1][:, -1, :] for r in rows]).contiguous().to(self.device)
                else:
                    shape = (B, kd.n_kv_heads, kd.head_dim)
                    k_new = values.normal(shape, kd.dtype, self.cfg.value_sigma, self.seed, 5, layer, k).to(self.device)
                    v_new = values.normal(shape, kd.dtype, self.cfg.value_sigma, self.seed, 6, layer, k).to(self.device)
            self.inputs[(k, layer)] = (q, k_new, v_new)
            self.out[(k, layer)] = torch.empty(B, kd.n_q_heads, kd.head_dim, dtype=torch.float32,
                                               device=self.device)

    # ---- device side of the step -------------------------------------------------
    def scale(self, k: int) -> float:
        return 1.0 / math.sqrt(self.cfg.kinds[k].head_dim)

    def run_layer(self, k: int, layer: int, split: bool = False, events=None) -> None:
        kd = self.cfg.kinds[k]
        q, k_new, v_new = self.inputs[(k, layer)]
        fused = self.fuse_append and k_new is not None
        if k_new is not None and not fused:
            self.pool.kv_append(k, layer, k_new, v_new, self.tables[k], self.seq_lens[k])
        kn, vn = (k_new, v_new) if fused else (None, None)
        if not split and events is None:
            self.pool.paged_decode(k, layer, q, self.tables[k], self.seq_lens[k], self.max_len[k],
                                   kd.window, self.scale(k), self.workspace[k], self.out[(k, layer)],
                                   self.pages_per_split, kn, vn)
            return
        if events is not None:
            events[0].record()
        self.pool.paged_decode_partial(k, layer, q, self.tables[k], self.seq_lens[k], self.max_len[k],
                                       kd.window, self.scale(k), self.workspace[k], self.pages_per_split,
                                       kn, vn)
        if events is not None:
            events[1].record()
        self.pool.splitk_reduce(k, kd.n_q_heads, self.seq_lens[k], self.max_len[k], kd.window,
                                self.workspace[k], self.out[(k, layer)], self.pages_per_split)

    def device_step(self, events: Optional[Dict] = None) -> None:
        """kv_append + paged_decode for every attention layer, in model order."""
        for k, layer in self.schedule:
            self.run_layer(k, layer, events=None if events is None else events[(k, layer)])

    # ---- accounting -----------------------------------------------------------------
    def visible_tokens(self, k: int) -> np.ndarray:
        kd = self.cfg.kinds[k]
        L = self.seq_lens_host[k].astype(np.int64)
        return np.minimum(L, kd.window) if kd.window > 0 else L

    def kv_bytes_layer(self, k: int) -> int:
        """Algorithmic K/V bytes one layer of kind k reads in the step."""
        return int(self.visible_tokens(k).sum()) * self.cfg.kinds[k].bytes_per_token_per_layer

    def kv_bytes_step(self) -> int:
        return sum(self.kv_bytes_layer(k) for k, _ in self.schedule)

    def gather(self, k: int, layer: int, b: int):
        """Contiguous K, V of request b read back through the harness's own address map (CPU)."""
        kd = self.cfg.kinds[k]
        return layout.gather_request(self.pool_u8, kd, layer, self.tables_host[k][b].tolist(),
                                     int(self.seq_lens_host[k][b]))

    def close(self) -> None:
        self.pool.destroy()
