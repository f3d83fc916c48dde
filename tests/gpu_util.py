"""Helpers of the GPU parity tests: build device caches from the seeded generator through the library's
own append entry point, and build the matching host problem for the CPU oracle from the same generator.
No expected value ever comes from the GPU side."""
import numpy as np
import torch

import oracle
from paper_2603_04428_amd import binding as b
from paper_2603_04428_amd.workload import build_device_cache

DEV = "cuda"


def gpu_cache(w, poison=True, extra_blocks=1, tokens=None, param_format=0):
    """Device pools of workload w filled with tokens 0..final_len-1 of every agent via q4kv_append.
    param_format: 0 binary16, 1 bfloat16 scale / bias (the same numbers on both sides of the boundary)."""
    return build_device_cache(w, DEV, poison, extra_blocks, tokens, param_format)


def host_cache(w, tokens=None, param_format=0):
    """The same logical cache on the host, quantized by the oracle."""
    spec = oracle.make_spec(w.num_layers, w.num_q_heads, w.num_kv_heads, w.k_dim, w.v_dim, w.v_aliases_k,
                            param_format=param_format)
    table, nb = w.block_table()
    nan_bits = 0x7FC0 if param_format else 0x7E00
    kpool = oracle.Pool(spec, w.k_dim, nb, fill=nan_bits)
    vpool = None if w.v_aliases_k else oracle.Pool(spec, w.v_dim, nb, fill=nan_bits)
    table = np.where(table < 0, 0, table).astype(np.int32)
    lens = w.final_lens() if tokens is None else tokens
    for a, n in enumerate(lens):
        if n == 0:
            continue
        k_new = np.stack([w.k_rows(l, a, 0, n).numpy() for l in range(w.num_layers)])[:, None]
        v_new = None if w.v_aliases_k else np.stack([w.v_rows(l, a, 0, n).numpy() for l in range(w.num_layers)])[:, None]
        oracle.append(spec, kpool, vpool, k_new, v_new, table[a:a + 1], np.zeros(1, np.int32))
    return spec, kpool, vpool, table


def oracle_unit(w, layer, agent, kvh, n, sm_scale=None, window=0, q=None, q_len=1, param_format=0):
    """Oracle attention of one (layer, agent, kv head) of a big workload, rebuilt alone on the host:
    returns float16 [q_len][n_rep][v_dim]."""
    R = w.n_rep
    alias = w.v_aliases_k
    spec = oracle.make_spec(1, R, 1, w.k_dim, w.v_dim, alias, param_format=param_format)
    nb = (n + 255) // 256
    kpool = oracle.Pool(spec, w.k_dim, max(nb, 1))
    vpool = None if alias else oracle.Pool(spec, w.v_dim, max(nb, 1))
    table = np.arange(max(nb, 1), dtype=np.int32)[None]
    k_new = w.k_rows(layer, agent, 0, n, h0=kvh, h1=kvh + 1).numpy()[None, None]
    v_new = None if alias else w.v_rows(layer, agent, 0, n, h0=kvh, h1=kvh + 1).numpy()[None, None]
    oracle.append(spec, kpool, vpool, k_new, v_new, table, np.zeros(1, np.int32))
    if q is None:
        q = w.q_rows(layer, agent).numpy()
    qh = np.ascontiguousarray(q[:, kvh * R:(kvh + 1) * R])[None, None]
    out = oracle.attention(spec, kpool, vpool, qh, table, [n], w.sm_scale if sm_scale is None else sm_scale,
                           window=window)
    return out[0, 0]


def bits(t):
    """device int32/int16/float16 tensor -> host numpy array of unsigned bit patterns"""
    a = t.cpu().numpy()
    return a.view({np.dtype(np.int32): np.uint32, np.dtype(np.int16): np.uint16,
                   np.dtype(np.float16): np.uint16}[a.dtype])
