"""Test-side helpers: call the oracle on a workload, brute-force references."""
import math

import numpy as np

from paper_2504_07494_amd import workloads as wl


def oracle_shape(o, batch, scale=None):
    c = batch.cfg
    return o.shape_of(c.d_model, c.n_heads, c.head_dim, c.block_size, c.dtype, batch.max_blocks,
                      c.softmax_scale if scale is None else scale)


def oracle_attn(o, batch, layer, pairs=None, want_weights=False, scale=None, kinds=None):
    return o.attn(oracle_shape(o, batch, scale), layer.q, layer.pool, layer.pool, layer.pool,
                  layer.W_K, layer.b_K, layer.W_V, layer.b_V, batch.block_tables, batch.ctx_lens,
                  batch.cache_kind if kinds is None else kinds, pairs=pairs, want_weights=want_weights)


def logical_kv(batch, layer, r):
    """(K, V) float64 [n][H][hd] of request r by the textbook definition, with numpy."""
    c = batch.cfg
    n = int(batch.ctx_lens[r])
    if batch.cache_kind[r] == wl.KIND_KV:
        K = np.stack([wl.to_f64(wl.kv_row_view(batch, layer.pool, r, j, 0), c.dtype) for j in range(n)])
        V = np.stack([wl.to_f64(wl.kv_row_view(batch, layer.pool, r, j, 1), c.dtype) for j in range(n)])
        return K, V
    X = np.stack([wl.to_f64(wl.hidden_row_view(batch, layer.pool, r, j), c.dtype) for j in range(n)])
    K = X @ wl.to_f64(layer.W_K, c.dtype) + wl.to_f64(layer.b_K, c.dtype)
    V = X @ wl.to_f64(layer.W_V, c.dtype) + wl.to_f64(layer.b_V, c.dtype)
    return K.reshape(n, c.n_heads, c.head_dim), V.reshape(n, c.n_heads, c.head_dim)


def brute_force_attention(q, K, V, scale):
    """Eq. 2-3 with explicit loops, no max subtraction.  q [hd], K, V [n][hd]."""
    n, hd = len(K), len(q)
    e = []
    for j in range(n):
        dot = 0.0
        for c in range(hd):
            dot += float(q[c]) * float(K[j][c])
        e.append(math.exp(dot * scale))
    den = 0.0
    for j in range(n):
        den += e[j]
    out = [0.0] * hd
    for j in range(n):
        for c in range(hd):
            out[c] += (e[j] / den) * float(V[j][c])
    return np.array(out)
