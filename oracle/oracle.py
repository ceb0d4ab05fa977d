"""ctypes loader of the C oracle.  TEST INFRASTRUCTURE ONLY."""
import ctypes as C
import os

import numpy as np

from . import build as _build

DTYPE_CODES = {"f32": 0, "f16": 1, "bf16": 2}


class OracleShape(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("block_size", C.c_int32), ("dtype", C.c_int32), ("max_blocks", C.c_int32),
                ("scale", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        # APT_ORACLE_LIB: a test loads a deliberately altered build of the oracle (mutation check of the pins)
        path = os.environ.get("APT_ORACLE_LIB") or _build.build(force=False)
        _lib = C.CDLL(path)
        _lib.apt_oracle_threads.restype = C.c_int
        for name in ("apt_oracle_attn", "apt_oracle_partial", "apt_oracle_merge", "apt_oracle_append"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def threads() -> int:
    return lib().apt_oracle_threads()


def shape_of(d_model, n_heads, head_dim, block_size, dtype, max_blocks, scale) -> OracleShape:
    return OracleShape(d_model, n_heads, head_dim, block_size, DTYPE_CODES[dtype], max_blocks, float(scale))


def attn(shape, q, k_pages, v_pages, hidden_pages, W_K, b_K, W_V, b_V, block_tables, ctx_lens, cache_kind,
         pairs=None, want_weights=False):
    """Attention output, double [n_pairs][head_dim] (all B*H pairs in [r][h] order if
    pairs is None).  With want_weights also the list of softmax weight vectors."""
    B = len(ctx_lens)
    H, hd = shape.n_heads, shape.head_dim
    ctx_lens = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    cache_kind = np.ascontiguousarray(cache_kind, dtype=np.uint8)
    block_tables = np.ascontiguousarray(block_tables, dtype=np.int32)
    assert block_tables.shape == (B, 2, shape.max_blocks)
    if pairs is None:
        sel_r = sel_h = None
        n_sel = B * H
        rs = np.repeat(np.arange(B), H)
    else:
        pairs = np.asarray(pairs, dtype=np.int32).reshape(-1, 2)
        sel_r = np.ascontiguousarray(pairs[:, 0])
        sel_h = np.ascontiguousarray(pairs[:, 1])
        n_sel = len(pairs)
        rs = sel_r
    out = np.empty((n_sel, hd), dtype=np.float64)
    w = None
    if want_weights:
        w = np.empty(int(ctx_lens[rs].astype(np.int64).sum()), dtype=np.float64)
    rc = lib().apt_oracle_attn(C.byref(shape), C.c_int(B), _p(q), _p(k_pages), _p(v_pages), _p(hidden_pages),
                               _p(W_K), _p(b_K), _p(W_V), _p(b_V), _p(block_tables), _p(ctx_lens),
                               _p(cache_kind), _p(sel_r), _p(sel_h), C.c_int(n_sel), _p(out), _p(w))
    if rc != 0:
        raise ValueError("apt_oracle_attn: bad argument")
    if want_weights:
        offs = np.concatenate([[0], np.cumsum(ctx_lens[rs].astype(np.int64))])
        return out, [w[offs[i]:offs[i + 1]] for i in range(n_sel)]
    return out


def partial(shape, q, k_pages, v_pages, hidden_pages, W_K, b_K, W_V, b_V, block_tables, kind, r, h, t0, t1):
    block_tables = np.ascontiguousarray(block_tables, dtype=np.int32)
    m = C.c_double()
    l = C.c_double()
    acc = np.empty(shape.head_dim, dtype=np.float64)
    rc = lib().apt_oracle_partial(C.byref(shape), _p(q), _p(k_pages), _p(v_pages), _p(hidden_pages),
                                  _p(W_K), _p(b_K), _p(W_V), _p(b_V), _p(block_tables),
                                  C.c_int(int(kind)), C.c_int(r), C.c_int(h), C.c_int(t0), C.c_int(t1),
                                  C.byref(m), C.byref(l), _p(acc))
    if rc != 0:
        raise ValueError("apt_oracle_partial: bad argument")
    return m.value, l.value, acc


def merge(m, l, acc):
    m = np.ascontiguousarray(m, dtype=np.float64)
    l = np.ascontiguousarray(l, dtype=np.float64)
    acc = np.ascontiguousarray(acc, dtype=np.float64)
    n, hd = acc.shape
    out = np.empty(hd, dtype=np.float64)
    rc = lib().apt_oracle_merge(C.c_int(n), C.c_int(hd), _p(m), _p(l), _p(acc), _p(out))
    if rc != 0:
        raise ValueError("apt_oracle_merge: bad argument")
    return out


def append(shape, x_new, k_new, v_new, k_pages, v_pages, hidden_pages, block_tables, ctx_lens, cache_kind):
    """In-place cache append of the current token's vectors (position ctx_lens[r] - 1)."""
    ctx_lens = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    cache_kind = np.ascontiguousarray(cache_kind, dtype=np.uint8)
    block_tables = np.ascontiguousarray(block_tables, dtype=np.int32)
    rc = lib().apt_oracle_append(C.byref(shape), C.c_int(len(ctx_lens)), _p(x_new), _p(k_new), _p(v_new),
                                 _p(k_pages), _p(v_pages), _p(hidden_pages), _p(block_tables), _p(ctx_lens),
                                 _p(cache_kind))
    if rc != 0:
        raise ValueError("apt_oracle_append: bad argument")


def write(shape, new_offsets, x_new, k_new, v_new, k_pages, v_pages, hidden_pages, block_tables, ctx_lens, cache_kind):
    """In-place cache write of runs of new tokens (positions ctx_lens[r] - n_r .. ctx_lens[r] - 1)."""
    ctx_lens = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    cache_kind = np.ascontiguousarray(cache_kind, dtype=np.uint8)
    block_tables = np.ascontiguousarray(block_tables, dtype=np.int32)
    new_offsets = np.ascontiguousarray(new_offsets, dtype=np.int32)
    rc = lib().apt_oracle_write(C.byref(shape), C.c_int(len(ctx_lens)), _p(new_offsets), _p(x_new), _p(k_new), _p(v_new),
                                _p(k_pages), _p(v_pages), _p(hidden_pages), _p(block_tables), _p(ctx_lens),
                                _p(cache_kind))
    if rc != 0:
        raise ValueError("apt_oracle_write: bad argument")
