"""ctypes binding of libapt_hybrid.so: the same names as include/apt_hybrid.h.

Argument marshalling only.  Device buffers are torch tensors (or raw integer
addresses); host buffers are numpy arrays.  Every computation runs in the
library's HIP kernels; there is no fallback: if the library has not been built
(python paper_2504_07494_amd/build.py, or __graft_entry__.build()), loading
raises.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libapt_hybrid.so")

APT_F32, APT_F16, APT_BF16 = 0, 1, 2
APT_KIND_KV, APT_KIND_HIDDEN = 0, 1
APT_HIDDEN_AUTO, APT_HIDDEN_VALU, APT_HIDDEN_MFMA, APT_HIDDEN_ABSORBED = 0, 1, 2, 3
APT_OK, APT_EINVAL, APT_ESHAPE, APT_EDTYPE, APT_EWORKSPACE, APT_EHIP, APT_ERANGE, APT_EFULL = 0, -1, -2, -3, -4, -5, -6, -7
DTYPE_CODES = {"f32": APT_F32, "f16": APT_F16, "bf16": APT_BF16}

# include/apt_hybrid.h (the product interface) and include/apt_hybrid_bench.h (measurement tooling)
EXPORTS = ["apt_strerror", "apt_version", "apt_init", "apt_workspace_bytes", "apt_plan_max_bytes", "apt_plan",
           "apt_plan_get_info", "apt_plan_upload", "apt_validate_host", "apt_packed_weight_bytes", "apt_pack_weights",
           "apt_hybrid_decode_attn", "apt_hybrid_decode_attn_static", "apt_cache_append", "apt_cache_write",
           "apt_pool_create", "apt_pool_destroy", "apt_pool_free_blocks", "apt_pool_blocks_needed", "apt_pool_assign",
           "apt_pool_extend", "apt_pool_release", "apt_pool_switch_kind", "apt_pool_export", "apt_schedule"]
BENCH_EXPORTS = ["apt_hybrid_decode_attn_timed", "apt_copy_bytes", "apt_probe_mfma"]


class apt_shape(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32), ("block_size", C.c_int32),
                ("dtype", C.c_int32), ("out_dtype", C.c_int32), ("max_blocks_per_req", C.c_int32),
                ("hidden_chunk", C.c_int32), ("kv_chunk", C.c_int32), ("hidden_impl", C.c_int32),
                ("softmax_scale", C.c_float), ("reserved", C.c_int32)]


class apt_plan_info(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_items", C.c_int32), ("n_hidden_items", C.c_int32),
                ("n_partials", C.c_int32), ("hidden_chunk", C.c_int32), ("kv_chunk", C.c_int32),
                ("hidden_impl", C.c_int32), ("reserved", C.c_int32), ("total_tokens", C.c_int64),
                ("hidden_tokens", C.c_int64), ("plan_bytes", C.c_uint64), ("workspace_bytes", C.c_uint64)]


class AptError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {apt_strerror(status)} ({status})")


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python paper_2504_07494_amd/build.py` "
                               "(there is no CPU fallback)")
        _lib = C.CDLL(LIB_PATH)
        _lib.apt_strerror.restype = C.c_char_p
        _lib.apt_strerror.argtypes = [C.c_int]
        for name in EXPORTS[1:] + BENCH_EXPORTS:
            getattr(_lib, name).restype = C.c_int
        _lib.apt_pool_destroy.restype = None
    return _lib


def _ptr(x):
    """Address of a torch tensor, numpy array, ctypes object or plain int (None -> NULL)."""
    if x is None:
        return C.c_void_p(None)
    if isinstance(x, C.c_void_p):
        return x
    if isinstance(x, int):
        return C.c_void_p(x)
    if isinstance(x, np.ndarray):
        return C.c_void_p(x.ctypes.data)
    if hasattr(x, "data_ptr"):
        return C.c_void_p(x.data_ptr())
    return C.cast(C.byref(x), C.c_void_p)


def _check(rc, where):
    if rc != APT_OK:
        raise AptError(rc, where)


def apt_strerror(status: int) -> str:
    return lib().apt_strerror(int(status)).decode()


def apt_version() -> int:
    return lib().apt_version()


def make_shape(d_model, n_heads, head_dim, block_size, dtype, max_blocks_per_req, softmax_scale,
               out_dtype="f32", hidden_chunk=0, kv_chunk=0, hidden_impl=APT_HIDDEN_AUTO) -> apt_shape:
    return apt_shape(d_model, n_heads, head_dim, block_size, DTYPE_CODES[dtype], DTYPE_CODES[out_dtype],
                     max_blocks_per_req, hidden_chunk, kv_chunk, hidden_impl, float(softmax_scale), 0)


def apt_init():
    _check(lib().apt_init(), "apt_init")


def apt_workspace_bytes(shape, max_batch, max_ctx):
    """Returns (dev_bytes, host_bytes)."""
    dev, host = C.c_size_t(), C.c_size_t()
    _check(lib().apt_workspace_bytes(C.byref(shape), C.c_int(max_batch), C.c_int(max_ctx), C.byref(dev), C.byref(host)),
           "apt_workspace_bytes")
    return dev.value, host.value


def apt_plan_max_bytes(shape, B, max_ctx) -> int:
    n = C.c_size_t()
    _check(lib().apt_plan_max_bytes(C.byref(shape), C.c_int(B), C.c_int(max_ctx), C.byref(n)), "apt_plan_max_bytes")
    return n.value


def apt_plan(shape, ctx_lens_host: np.ndarray, cache_kind_host: np.ndarray, plan_host) -> apt_plan_info:
    """plan_host: numpy int32 array or page-locked torch int32 CPU tensor that receives the blob."""
    assert ctx_lens_host.dtype == np.int32 and cache_kind_host.dtype == np.uint8
    info = apt_plan_info()
    nbytes = plan_host.nbytes if isinstance(plan_host, np.ndarray) else plan_host.numel() * plan_host.element_size()
    _check(lib().apt_plan(C.byref(shape), _ptr(ctx_lens_host), _ptr(cache_kind_host), C.c_int(len(ctx_lens_host)),
                          _ptr(plan_host), C.c_size_t(nbytes), C.byref(info)), "apt_plan")
    return info


def apt_plan_get_info(plan_host) -> apt_plan_info:
    info = apt_plan_info()
    _check(lib().apt_plan_get_info(_ptr(plan_host), C.byref(info)), "apt_plan_get_info")
    return info


def apt_plan_upload(plan_host, plan_dev, stream=0):
    _check(lib().apt_plan_upload(_ptr(plan_host), _ptr(plan_dev), C.c_void_p(stream)), "apt_plan_upload")


def apt_validate_host(shape, ctx_lens_host, cache_kind_host, block_tables_host, n_pool_blocks):
    _check(lib().apt_validate_host(C.byref(shape), _ptr(ctx_lens_host), _ptr(cache_kind_host),
                                   _ptr(block_tables_host), C.c_int(len(ctx_lens_host)),
                                   C.c_int64(n_pool_blocks)), "apt_validate_host")


def apt_packed_weight_bytes(shape) -> int:
    n = C.c_size_t()
    _check(lib().apt_packed_weight_bytes(C.byref(shape), C.byref(n)), "apt_packed_weight_bytes")
    return n.value


def apt_pack_weights(shape, W_K, W_V, packed, stream=0):
    _check(lib().apt_pack_weights(C.byref(shape), _ptr(W_K), _ptr(W_V), _ptr(packed), C.c_void_p(stream)),
           "apt_pack_weights")


def apt_hybrid_decode_attn(shape, plan_host, plan_dev, q, k_pages, v_pages, hidden_pages, W_K, W_V, W_packed,
                           b_K, b_V, block_tables, out, workspace, workspace_bytes, stream=0):
    _check(lib().apt_hybrid_decode_attn(C.byref(shape), _ptr(plan_host), _ptr(plan_dev), _ptr(q), _ptr(k_pages),
                                        _ptr(v_pages), _ptr(hidden_pages), _ptr(W_K), _ptr(W_V), _ptr(W_packed),
                                        _ptr(b_K), _ptr(b_V), _ptr(block_tables), _ptr(out), _ptr(workspace),
                                        C.c_size_t(workspace_bytes), C.c_void_p(stream)), "apt_hybrid_decode_attn")


APT_STATIC_WORKSPACE_BYTES = 64 << 20


def apt_hybrid_decode_attn_static(shape, plan_host, plan_dev, q, k_pages, v_pages, hidden_pages, W_K, W_V, W_packed,
                                  b_K, b_V, block_tables, out, stream=0):
    _check(lib().apt_hybrid_decode_attn_static(C.byref(shape), _ptr(plan_host), _ptr(plan_dev), _ptr(q), _ptr(k_pages),
                                               _ptr(v_pages), _ptr(hidden_pages), _ptr(W_K), _ptr(W_V), _ptr(W_packed),
                                               _ptr(b_K), _ptr(b_V), _ptr(block_tables), _ptr(out), C.c_void_p(stream)),
           "apt_hybrid_decode_attn_static")


def apt_hybrid_decode_attn_timed(shape, plan_host, plan_dev, q, k_pages, v_pages, hidden_pages, W_K, W_V, W_packed,
                                 b_K, b_V, block_tables, out, workspace, workspace_bytes, stream, ev_begin, ev_end):
    """ev_begin / ev_end: raw hipEvent_t handles (int) or None."""
    _check(lib().apt_hybrid_decode_attn_timed(C.byref(shape), _ptr(plan_host), _ptr(plan_dev), _ptr(q),
                                              _ptr(k_pages), _ptr(v_pages), _ptr(hidden_pages), _ptr(W_K), _ptr(W_V),
                                              _ptr(W_packed), _ptr(b_K), _ptr(b_V), _ptr(block_tables), _ptr(out),
                                              _ptr(workspace), C.c_size_t(workspace_bytes), C.c_void_p(stream),
                                              _ptr(ev_begin), _ptr(ev_end)), "apt_hybrid_decode_attn_timed")


def apt_cache_append(shape, B, x_new, k_new, v_new, k_pages, v_pages, hidden_pages, block_tables, ctx_lens_dev,
                     cache_kind_dev, stream=0):
    _check(lib().apt_cache_append(C.byref(shape), C.c_int(B), _ptr(x_new), _ptr(k_new), _ptr(v_new), _ptr(k_pages),
                                  _ptr(v_pages), _ptr(hidden_pages), _ptr(block_tables), _ptr(ctx_lens_dev),
                                  _ptr(cache_kind_dev), C.c_void_p(stream)), "apt_cache_append")


def apt_cache_write(shape, B, new_offsets_dev, max_new_tokens, x_new, k_new, v_new, k_pages, v_pages, hidden_pages,
                    block_tables, ctx_lens_dev, cache_kind_dev, stream=0):
    _check(lib().apt_cache_write(C.byref(shape), C.c_int(B), _ptr(new_offsets_dev), C.c_int32(max_new_tokens),
                                 _ptr(x_new), _ptr(k_new), _ptr(v_new), _ptr(k_pages), _ptr(v_pages),
                                 _ptr(hidden_pages), _ptr(block_tables), _ptr(ctx_lens_dev), _ptr(cache_kind_dev),
                                 C.c_void_p(stream)), "apt_cache_write")


# --- hybrid cache assigner (host-side pool bookkeeping); `pool` is the opaque handle --------------
def apt_pool_create(n_blocks, block_size, max_blocks_per_req, max_requests) -> C.c_void_p:
    h = C.c_void_p()
    _check(lib().apt_pool_create(C.c_int64(n_blocks), C.c_int32(block_size), C.c_int32(max_blocks_per_req),
                                 C.c_int32(max_requests), C.byref(h)), "apt_pool_create")
    return h


def apt_pool_destroy(pool):
    lib().apt_pool_destroy(pool)


def apt_pool_free_blocks(pool) -> int:
    n = C.c_int64()
    _check(lib().apt_pool_free_blocks(pool, C.byref(n)), "apt_pool_free_blocks")
    return n.value


def apt_pool_blocks_needed(pool, kind, n_tokens) -> int:
    n = C.c_int64()
    _check(lib().apt_pool_blocks_needed(pool, C.c_uint8(kind), C.c_int32(n_tokens), C.byref(n)), "apt_pool_blocks_needed")
    return n.value


def apt_pool_assign(pool, slot, kind, n_tokens):
    _check(lib().apt_pool_assign(pool, C.c_int32(slot), C.c_uint8(kind), C.c_int32(n_tokens)), "apt_pool_assign")


def apt_pool_extend(pool, slot, n_tokens):
    _check(lib().apt_pool_extend(pool, C.c_int32(slot), C.c_int32(n_tokens)), "apt_pool_extend")


def apt_pool_release(pool, slot):
    _check(lib().apt_pool_release(pool, C.c_int32(slot)), "apt_pool_release")


def apt_pool_switch_kind(pool, slot, new_kind):
    _check(lib().apt_pool_switch_kind(pool, C.c_int32(slot), C.c_uint8(new_kind)), "apt_pool_switch_kind")


def apt_pool_export(pool, slots: np.ndarray, block_tables: np.ndarray, ctx_lens: np.ndarray, cache_kind: np.ndarray):
    """Fills the host arrays block_tables int32 [B][2][max_blocks], ctx_lens int32 [B], cache_kind uint8 [B]."""
    assert slots.dtype == np.int32 and block_tables.dtype == np.int32 and ctx_lens.dtype == np.int32
    assert cache_kind.dtype == np.uint8
    _check(lib().apt_pool_export(pool, _ptr(slots), C.c_int(len(slots)), _ptr(block_tables), _ptr(ctx_lens),
                                 _ptr(cache_kind)), "apt_pool_export")


def apt_schedule(pending: np.ndarray, mem: np.ndarray, mem_limit, n_unfinished, rho):
    """Returns (alpha uint8 [n], beta uint8 [n], value)."""
    assert pending.dtype == np.float64 and mem.dtype == np.int64 and len(pending) == len(mem)
    alpha = np.empty(len(pending), dtype=np.uint8)
    beta = np.empty(len(pending), dtype=np.uint8)
    val = C.c_double()
    _check(lib().apt_schedule(_ptr(pending), _ptr(mem), C.c_int(len(pending)), C.c_int64(mem_limit),
                              C.c_int32(n_unfinished), C.c_double(rho), _ptr(alpha), _ptr(beta), C.byref(val)),
           "apt_schedule")
    return alpha, beta, val.value


def apt_copy_bytes(dst, src, nbytes, stream=0):
    _check(lib().apt_copy_bytes(_ptr(dst), _ptr(src), C.c_size_t(nbytes), C.c_void_p(stream)), "apt_copy_bytes")


def apt_probe_mfma(out, n_workgroups, iters, random_operands=0, variant=0, stream=0):
    _check(lib().apt_probe_mfma(_ptr(out), C.c_int(n_workgroups), C.c_int(iters), C.c_int(random_operands),
                                C.c_int(variant), C.c_void_p(stream)), "apt_probe_mfma")


# --- decoding of a plan blob for tests (layout documented in the header) ------------------
def decode_plan(plan_host) -> dict:
    w = plan_host if isinstance(plan_host, np.ndarray) else plan_host.numpy()
    w = w.view(np.int32).reshape(-1)
    B, n_items, off = int(w[1]), int(w[3]), int(w[9])
    return {
        "split_count": w[32:32 + B].tolist(),
        "ws_offset": w[32 + B:32 + 2 * B].tolist(),
        "queue_offset": w[16:25].tolist(),
        "items": [tuple(int(v) for v in row) for row in w[off:off + 4 * n_items].reshape(n_items, 4)],
        "n_hidden_items": int(w[4]),
        "n_partials": int(w[5]),
    }
