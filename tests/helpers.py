"""Glue shared by the tests: the same workload config instantiated on the oracle and on the library."""
from __future__ import annotations

import numpy as np

from oracle.alloc import OraclePool, OracleRequests, lcm_bytes
from workloads import configs, scripts

import paper_2503_18292_amd as J
from paper_2503_18292_amd.api import make_kind

TYPE = {configs.FULL: J.FULL, configs.WINDOW: J.WINDOW, configs.CROSS: J.CROSS, configs.OPAQUE: J.OPAQUE}
DTYPE = {"f32": J.F32, "bf16": J.BF16}


def kind_descs(cfg):
    out = []
    for k in cfg.kinds:
        if k.type == configs.OPAQUE:
            out.append(make_kind(J.OPAQUE, DTYPE[k.dtype], k.n_layers, 0, 0, 1, 0, k.small_page_bytes))
        else:
            out.append(make_kind(TYPE[k.type], DTYPE[k.dtype], k.n_layers, k.n_kv_heads, k.head_dim,
                                 k.tokens_per_page, k.window, 0))
    return out


def large_pages_for(cfg, ctx):
    S = [k.small_page_bytes for k in cfg.kinds]
    if cfg.pool_large_pages is not None:
        return cfg.pool_large_pages
    return scripts.pool_large_pages_needed(cfg, ctx, lcm_bytes(S))


def make_oracle(cfg, n_large):
    S = [k.small_page_bytes for k in cfg.kinds]
    pool = OraclePool(n_large * lcm_bytes(S), S)
    reqs = OracleRequests(pool, [k.tokens_per_page for k in cfg.kinds], [k.window for k in cfg.kinds])
    return pool, reqs


def make_library(cfg, n_large, device_base=None):
    descs = kind_descs(cfg)
    return J.Pool(device_base, n_large * J.lcm_page_bytes(descs), descs)


def table_width(cfg, kind_index, ctx):
    k = cfg.kinds[kind_index]
    if k.type == configs.CROSS:
        n = cfg.cross_len
    elif k.type == configs.OPAQUE:
        n = 1
    else:
        n = int(np.max(ctx)) + 1
    return -(-n // k.tokens_per_page)


def oracle_table(reqs, cfg, kind_index, width):
    return np.array([reqs.row(scripts.request_id(b), kind_index, width) for b in range(cfg.batch)],
                    dtype=np.int32)


def library_table(pool, cfg, kind_index, width):
    return pool.block_table([scripts.request_id(b) for b in range(cfg.batch)], kind_index, width).numpy()
