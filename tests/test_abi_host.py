"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, the
host planner matches the plain partition rule bit for bit, and bad arguments are turned
into error codes.  No device call is made here."""
import os
import re

import numpy as np
import pytest

from oracle import plan_oracle as po
from paper_2504_07494_amd import binding as ab

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _shape(**kw):
    base = dict(d_model=5120, n_heads=40, head_dim=128, block_size=16, dtype="f16", max_blocks_per_req=128,
                softmax_scale=128 ** -0.5)
    base.update(kw)
    return ab.make_shape(**base)


def _declared(header_name):
    header = open(os.path.join(ROOT, "include", header_name)).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)          # declarations only, not the prose about them
    return set(re.findall(r"\b(apt_[a-z_0-9]+)\s*\(", header))


def test_library_exports_every_declared_symbol():
    declared = _declared("apt_hybrid.h")
    assert declared == set(ab.EXPORTS), declared ^ set(ab.EXPORTS)
    bench = _declared("apt_hybrid_bench.h")
    assert bench == set(ab.BENCH_EXPORTS), bench ^ set(ab.BENCH_EXPORTS)
    lib = ab.lib()
    for name in declared | bench:
        assert hasattr(lib, name), name
    assert ab.apt_version() >= 100
    assert ab.apt_strerror(0) == "ok" and "shape" in ab.apt_strerror(ab.APT_ESHAPE)


@pytest.mark.parametrize("himpl", [ab.APT_HIDDEN_AUTO, ab.APT_HIDDEN_VALU, ab.APT_HIDDEN_MFMA, ab.APT_HIDDEN_ABSORBED])
def test_workspace_bound_covers_every_batch(himpl):
    """apt_workspace_bytes(max_batch, max_ctx) is at least what any batch within those limits needs, for every
    mix of the two cache kinds, and the all-one-kind extremes show that it is not a loose guess."""
    g = np.random.default_rng(11 + himpl)
    for kw in (dict(), dict(d_model=9216, n_heads=72), dict(d_model=256, n_heads=4, head_dim=64, dtype="f32")):
        if himpl == ab.APT_HIDDEN_MFMA and kw.get("dtype") == "f32":
            continue
        shape = _shape(hidden_impl=himpl, **kw)
        max_batch, max_ctx = 48, 2048
        dev, host = ab.apt_workspace_bytes(shape, max_batch, max_ctx)
        assert host == ab.apt_plan_max_bytes(shape, max_batch, max_ctx)
        worst = 0
        for trial in range(30):
            B = int(g.integers(1, max_batch + 1)) if trial else max_batch
            lens = g.integers(1, max_ctx + 1, size=B) if trial > 2 else np.full(B, max_ctx)
            ratio = [1.0, 0.0, 0.5][trial] if trial < 3 else g.random()
            kinds = (g.random(B) < ratio).astype(np.uint8)
            buf, info = _plan(shape, lens, kinds)
            assert info.workspace_bytes <= dev and info.plan_bytes <= host
            worst = max(worst, int(info.workspace_bytes))
        assert worst >= 0.5 * dev
    with pytest.raises(ab.AptError) as e:
        ab.apt_workspace_bytes(_shape(), 0, 100)
    assert e.value.status == ab.APT_EINVAL
    with pytest.raises(ab.AptError) as e:
        ab.apt_workspace_bytes(_shape(), 4, 128 * 16 + 1)
    assert e.value.status == ab.APT_ERANGE


def test_validate_host_rejects_a_hidden_pool_beyond_the_mfma_kernels_offset_range():
    shape = _shape()                                   # block = 16 * 5120 * 2 B = 160 KiB; 64 GiB = 419430.4 blocks
    lens, kinds = np.array([20], dtype=np.int32), np.array([1], dtype=np.uint8)
    bt = np.zeros((1, 2, 128), dtype=np.int32)
    ab.apt_validate_host(shape, lens, kinds, bt, 419430)
    with pytest.raises(ab.AptError) as e:
        ab.apt_validate_host(shape, lens, kinds, bt, 419431)
    assert e.value.status == ab.APT_ERANGE
    ab.apt_validate_host(_shape(hidden_impl=ab.APT_HIDDEN_ABSORBED), lens, kinds, bt, 419431)


def test_mfma_tile_default_follows_d_model_and_both_tiles_can_be_asked_for():
    for kw, want in ((dict(), 256), (dict(d_model=9216, n_heads=72), 320), (dict(hidden_chunk=320), 320),
                     (dict(d_model=9216, n_heads=72, hidden_chunk=256), 256)):
        buf, info = _plan(_shape(**kw), [700, 30], [1, 1])
        assert info.hidden_impl == ab.APT_HIDDEN_MFMA and info.hidden_chunk == want
        assert info.n_partials == sum(-(-n // want) for n in (700, 30))


def _plan(shape, lens, kinds):
    lens = np.asarray(lens, dtype=np.int32)
    kinds = np.asarray(kinds, dtype=np.uint8)
    nbytes = ab.apt_plan_max_bytes(shape, len(lens), int(lens.max()))
    buf = np.full(nbytes // 4, -7, dtype=np.int32)
    info = ab.apt_plan(shape, lens, kinds, buf)
    return buf, info


@pytest.mark.parametrize("seed,B,lo,hi,ratio", [(0, 64, 128, 2048, 0.5), (1, 1, 1, 1, 1.0), (2, 33, 1, 700, 0.3),
                                                (3, 256, 64, 2048, 0.0), (4, 17, 255, 258, 1.0)])
def test_plan_is_bit_exact_against_the_rule(seed, B, lo, hi, ratio):
    g = np.random.default_rng(seed)
    lens = g.integers(lo, hi + 1, size=B)
    kinds = (g.random(B) < ratio).astype(np.uint8)
    shape = _shape()
    buf, info = _plan(shape, lens, kinds)
    got = ab.decode_plan(buf)
    assert info.kv_chunk == po.auto_kv_chunk(lens, kinds, 40, 16)
    want = po.plan(lens, kinds, 40, info.hidden_chunk, info.kv_chunk)
    assert got == want
    assert info.n_items == len(want["items"]) and info.n_hidden_items == want["n_hidden_items"]
    assert info.n_partials == want["n_partials"]
    assert info.total_tokens == int(lens.sum()) and info.hidden_tokens == int(lens[kinds == 1].sum())
    assert info.workspace_bytes == want["n_partials"] * 40 * (128 + 2) * 4
    assert info.hidden_impl == ab.APT_HIDDEN_MFMA and info.hidden_chunk == 256
    # deterministic bytes
    buf2, _ = _plan(shape, lens, kinds)
    assert np.array_equal(buf[:info.plan_bytes // 4], buf2[:info.plan_bytes // 4])


def test_plan_with_explicit_chunks_and_small_heads():
    shape = _shape(d_model=256, n_heads=4, head_dim=64, dtype="f32", max_blocks_per_req=8, hidden_chunk=8, kv_chunk=32)
    lens, kinds = [16, 128, 1, 77], [1, 0, 1, 0]
    buf, info = _plan(shape, lens, kinds)
    assert info.hidden_impl == ab.APT_HIDDEN_VALU
    assert ab.decode_plan(buf) == po.plan(lens, kinds, 4, 8, 32)


def test_absorbed_plan_has_one_hidden_item_per_range_and_the_request_maps():
    g = np.random.default_rng(11)
    B = 37
    lens = g.integers(1, 2049, size=B)
    kinds = (g.random(B) < 0.5).astype(np.uint8)
    shape = _shape(hidden_impl=ab.APT_HIDDEN_ABSORBED)
    buf, info = _plan(shape, lens, kinds)
    assert info.hidden_impl == ab.APT_HIDDEN_ABSORBED and info.hidden_chunk == 512
    want = po.plan(lens, kinds, 40, 512, info.kv_chunk, hidden_item_per_head=False)
    assert ab.decode_plan(buf) == want
    # per-request maps of the hidden-kind requests, from their plain definitions
    w = buf.view(np.int32)
    arr = lambda i: w[32 + i * B:32 + (i + 1) * B].tolist()
    hid = [r for r in range(B) if kinds[r] == 1]
    assert arr(2) == kinds.tolist() and arr(3) == lens.tolist()
    assert arr(7) == hid + [-1] * (B - len(hid))
    tok = chunk = 0
    for i, r in enumerate(hid):
        assert (arr(4)[r], arr(5)[r], arr(6)[r]) == (i, tok, chunk)
        tok += int(lens[r])
        chunk += -(-int(lens[r]) // 512)
    assert all(arr(4)[r] == -1 for r in range(B) if kinds[r] == 0)
    # workspace: partials + QT + CB + S slices + (m, l) + YP + output partials, each section 256-byte aligned
    al = lambda v: (v + 255) // 256 * 256
    H, d, nh = 40, 5120, len(hid)
    end = want["n_partials"] * H * (128 + 2) * 4
    ks = d // 512
    for sec in (nh * d * 256, nh * H * 4, ks * tok * H * 4, nh * H * 8, chunk * H * d * 4, (d // 256) * nh * H * 128 * 4):
        end = al(end) + sec
    assert info.workspace_bytes == al(end) + chunk * 16 * 32 * 256
    for bad in (dict(n_heads=129, d_model=129 * 128), dict(n_heads=41, d_model=41 * 128, dtype="f32"), dict(hidden_chunk=256)):
        with pytest.raises(ab.AptError):
            _plan(_shape(hidden_impl=ab.APT_HIDDEN_ABSORBED, **bad), lens, kinds)


def test_plan_rejects_bad_arguments():
    shape = _shape()
    buf = np.zeros(1 << 16, dtype=np.int32)
    with pytest.raises(ab.AptError) as e:
        ab.apt_plan(shape, np.array([0], dtype=np.int32), np.array([0], dtype=np.uint8), buf)
    assert e.value.status == ab.APT_EINVAL
    with pytest.raises(ab.AptError) as e:
        ab.apt_plan(shape, np.array([5], dtype=np.int32), np.array([2], dtype=np.uint8), buf)
    assert e.value.status == ab.APT_EINVAL
    with pytest.raises(ab.AptError) as e:
        ab.apt_plan(shape, np.array([128 * 16 + 1], dtype=np.int32), np.array([0], dtype=np.uint8), buf)
    assert e.value.status == ab.APT_ERANGE
    with pytest.raises(ab.AptError) as e:
        ab.apt_plan(shape, np.array([2048] * 8, dtype=np.int32), np.array([1] * 8, dtype=np.uint8), buf[:64])
    assert e.value.status == ab.APT_EWORKSPACE


@pytest.mark.parametrize("kw,status", [
    (dict(n_heads=39), ab.APT_ESHAPE),                 # H * hd != d
    (dict(head_dim=96, n_heads=40, d_model=3840), ab.APT_ESHAPE),
    (dict(block_size=12), ab.APT_ESHAPE),
    (dict(hidden_chunk=128), ab.APT_ESHAPE),           # the MFMA tile is 256 or 320 tokens
    (dict(kv_chunk=100), ab.APT_ESHAPE),               # not a multiple of the block size
    (dict(dtype="f32", hidden_impl=ab.APT_HIDDEN_MFMA), ab.APT_ESHAPE),
    (dict(dtype="f16", out_dtype="bf16"), ab.APT_EDTYPE),
])
def test_shape_validation(kw, status):
    shape = _shape(**kw)
    with pytest.raises(ab.AptError) as e:
        ab.apt_plan_max_bytes(shape, 4, 100)
    assert e.value.status == status


def test_validate_host_range_checks_block_ids():
    shape = _shape(max_blocks_per_req=4)
    lens = np.array([20, 33], dtype=np.int32)
    kinds = np.array([0, 1], dtype=np.uint8)
    bt = np.full((2, 2, 4), -1, dtype=np.int32)
    bt[0, 0, :2] = [0, 1]; bt[0, 1, :2] = [2, 3]; bt[1, 0, :3] = [4, 5, 6]
    ab.apt_validate_host(shape, lens, kinds, bt, 7)
    with pytest.raises(ab.AptError) as e:
        ab.apt_validate_host(shape, lens, kinds, bt, 6)
    assert e.value.status == ab.APT_ERANGE
    bt[0, 1, 1] = -1
    with pytest.raises(ab.AptError):
        ab.apt_validate_host(shape, lens, kinds, bt, 7)


def test_kv_range_length_left_open_follows_the_batch():
    """kv_chunk = 0: the longest of 2048 / 1024 / 512 that still yields 2048 KV-kind items; hand-computed cases."""
    cases = [
        # (lens, kinds, heads, block size, chosen)
        ([2048] * 52, [0] * 52, 40, 16, 2048),               # 52 x 40 = 2080 items of 2048 tokens
        ([2048] * 51, [0] * 51, 40, 16, 1024),               # 2040 < 2048 at 2048, 4080 at 1024
        ([2048] * 25, [0] * 25, 40, 16, 512),                # 1000, 2000, then 4000 at 512
        ([2048] * 26, [0] * 26, 40, 16, 1024),               # 2080 at 1024
        ([16384], [0], 40, 16, 512),                         # one long request: 8 / 16 / 32 ranges x 40 heads
        ([2048] * 64, [1] * 64, 40, 16, 512),                # no KV-kind request
        ([2048] * 52 + [2048] * 100, [0] * 52 + [1] * 100, 40, 16, 2048),   # hidden-kind requests do not count
        ([2048] * 52, [0] * 52, 40, 4, 1024),                # 2048 tokens would be 512 blocks of 4: not allowed
        ([100] * 60, [0] * 60, 40, 16, 2048),                # short requests: one range each whatever the length
    ]
    for lens, kinds, H, bs, want in cases:
        mb = -(-max(lens) // bs)
        shape = _shape(d_model=H * 128, n_heads=H, block_size=bs, max_blocks_per_req=mb)
        _, info = _plan(shape, lens, kinds)
        assert info.kv_chunk == want == po.auto_kv_chunk(lens, kinds, H, bs), (lens[:2], len(lens), bs)
        # a length the caller fixes is taken as it is
        _, info = _plan(_shape(d_model=H * 128, n_heads=H, block_size=bs, max_blocks_per_req=mb, kv_chunk=512), lens, kinds)
        assert info.kv_chunk == 512


def test_attention_call_rejects_bad_arguments_before_any_launch():
    # null pointers and a foreign plan are caught on the host (no device is touched)
    shape = _shape()
    buf, info = _plan(shape, [300], [0])
    with pytest.raises(ab.AptError) as e:
        ab.apt_hybrid_decode_attn(shape, buf, None, None, None, None, None, None, None, None, None, None, None,
                                  None, None, 0)
    assert e.value.status == ab.APT_EINVAL
    for other in (_shape(kv_chunk=256), _shape(max_blocks_per_req=64), _shape(dtype="bf16"), _shape(block_size=32)):
        with pytest.raises(ab.AptError) as e:
            ab.apt_hybrid_decode_attn(other, buf, 16, 16, 16, 16, None, None, None, None, None, None, 16, 16, 16, 1 << 30)
        assert e.value.status == ab.APT_ESHAPE
    with pytest.raises(ab.AptError) as e:
        ab.apt_hybrid_decode_attn(shape, buf, 16, 16, 16, 16, None, None, None, None, None, None, 16, 16, 16, 8)
    assert e.value.status == ab.APT_EWORKSPACE


def test_static_workspace_call_rejects_bad_arguments_before_any_launch():
    # the entry point that allocates nothing validates like the ordinary one, and also refuses what its fixed
    # workspace cannot hold and the absorbed-weight path (no device is touched by any of these calls)
    shape = _shape()
    buf, info = _plan(shape, [300, 17], [0, 1])
    assert info.workspace_bytes <= ab.APT_STATIC_WORKSPACE_BYTES
    P = 16
    with pytest.raises(ab.AptError) as e:
        ab.apt_hybrid_decode_attn_static(shape, buf, None, None, None, None, None, None, None, None, None, None,
                                         None, None)
    assert e.value.status == ab.APT_EINVAL
    with pytest.raises(ab.AptError) as e:
        ab.apt_hybrid_decode_attn_static(_shape(block_size=32), buf, P, P, P, P, None, None, None, None, None, None, P, P)
    assert e.value.status == ab.APT_ESHAPE
    absorbed = _shape(hidden_impl=ab.APT_HIDDEN_ABSORBED)
    abuf, _ = _plan(absorbed, [300, 17], [0, 1])
    with pytest.raises(ab.AptError) as e:
        ab.apt_hybrid_decode_attn_static(absorbed, abuf, P, P, P, P, P, P, P, None, P, P, P, P)
    assert e.value.status == ab.APT_ESHAPE
    big = _shape(d_model=9216, n_heads=72, max_blocks_per_req=128)
    lens = [2048] * 512
    bbuf, binfo = _plan(big, lens, [1] * len(lens))
    assert binfo.workspace_bytes > ab.APT_STATIC_WORKSPACE_BYTES
    with pytest.raises(ab.AptError) as e:
        ab.apt_hybrid_decode_attn_static(big, bbuf, P, P, P, P, None, None, None, None, None, None, P, P)
    assert e.value.status == ab.APT_EWORKSPACE


def test_cache_write_calls_reject_bad_arguments_before_any_launch():
    shape = _shape()
    P = 16          # any non-null address: validation fails before a launch could use it
    for call in (lambda: ab.apt_cache_append(shape, 0, P, None, None, None, None, P, P, P, P),            # B < 1
                 lambda: ab.apt_cache_append(shape, 2, None, None, None, P, P, P, P, P, P),                # nothing to write
                 lambda: ab.apt_cache_append(shape, 2, P, None, None, None, None, None, P, P, P),          # x without its pool
                 lambda: ab.apt_cache_append(shape, 2, None, P, None, P, P, None, P, P, P),                # k without v
                 lambda: ab.apt_cache_append(shape, 2, None, P, P, P, None, None, P, P, P),                # v pool missing
                 lambda: ab.apt_cache_write(shape, 2, None, 4, P, None, None, None, None, P, P, P, P),     # no offsets
                 lambda: ab.apt_cache_write(shape, 2, P, 0, P, None, None, None, None, P, P, P, P),        # max_new_tokens < 1
                 lambda: ab.apt_cache_write(shape, 2, P, 4, P, None, None, None, None, P, None, P, P)):    # no block tables
        with pytest.raises(ab.AptError) as e:
            call()
        assert e.value.status == ab.APT_EINVAL
    with pytest.raises(ab.AptError) as e:
        ab.apt_cache_write(shape, 2, P, 8 * 65536, P, None, None, None, None, P, P, P, P)
    assert e.value.status == ab.APT_ERANGE
    with pytest.raises(ab.AptError) as e:
        ab.apt_cache_write(_shape(head_dim=96, d_model=96 * 40), 2, P, 4, P, None, None, None, None, P, P, P, P)
    assert e.value.status == ab.APT_ESHAPE
