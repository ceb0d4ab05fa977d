"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element
on the same seeded inputs.  Tolerance (fp16/bf16/fp32 in, fp32 accumulate): max-abs error
2e-3 and max-rel error 1e-2 (relative error over elements with |oracle| >= 1e-2)."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from paper_2504_07494_amd import binding as ab
from paper_2504_07494_amd import workloads as wl
from tests.helpers import oracle_attn

pytestmark = pytest.mark.gpu

MAX_ABS, MAX_REL = 2e-3, 1e-2
KV, HID = wl.KIND_KV, wl.KIND_HIDDEN


def _errors(got, want):
    err = np.abs(got - want)
    big = np.abs(want) >= 1e-2
    rel = float((err[big] / np.abs(want[big])).max()) if big.any() else 0.0
    return float(err.max()), rel


def _check(got, want, label, max_abs=MAX_ABS, max_rel=MAX_REL):
    assert np.all(np.isfinite(got)), f"{label}: non-finite output"
    a, r = _errors(got, want)
    print(f"[parity] {label}: max_abs={a:.3e} max_rel={r:.3e}", flush=True)
    assert a <= max_abs and r <= max_rel, f"{label}: max_abs={a:.3e} max_rel={r:.3e}"
    return a, r


def _run(batch, layer, **kw):
    from paper_2504_07494_amd.harness import DecodeRunner
    separate = kw.pop("separate_pools", False)
    rn = DecodeRunner(batch, **kw)
    dl = rn.upload(layer, separate_pools=separate)
    rn.run(dl)
    return rn, rn.out_f64()


def _full(oracle, batch, layer):
    c = batch.cfg
    return oracle_attn(oracle, batch, layer).reshape(batch.B, c.n_heads, c.head_dim)


def test_tiny_config_full_parity(oracle):
    print("[case] tiny config fp32", flush=True)
    batch = wl.make_batch(wl.CONFIGS["tiny"])
    layer = wl.make_layer(batch)
    rn, got = _run(batch, layer)
    assert rn.info.hidden_impl == ab.APT_HIDDEN_VALU
    _check(got, _full(oracle, batch, layer), "tiny", 1e-4, 1e-3)


MID = dict(d_model=512, n_heads=4, head_dim=128, block_size=16, batch=7, len_lo=1, len_hi=900, hidden_ratio=0.5)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("tile", [256, 320])
def test_mid_mfma_several_tiles_and_ragged_tails(oracle, dtype, tile):
    """Both token tiles of the MFMA kernel (256: all accumulators in AGPRs; 320: the fifth token block of a wave
    accumulated in VGPRs), with lengths around every tile and block boundary."""
    print(f"[case] mid mfma {dtype} tile {tile}", flush=True)
    cfg = wl.small_config(name="mid", dtype=dtype, **dict(MID, batch=12))
    lens = np.array([900, 257, 1, 512, 513, 256, 33, 319, 320, 321, 640, 289], dtype=np.int32)
    kinds = np.array([HID, HID, HID, KV, KV, HID, KV, HID, HID, HID, HID, HID], dtype=np.uint8)
    batch = wl.make_batch(cfg, lens, kinds)
    layer = wl.make_layer(batch)
    rn, got = _run(batch, layer, hidden_chunk=tile)
    assert rn.info.hidden_impl == ab.APT_HIDDEN_MFMA and rn.info.hidden_chunk == tile
    _check(got, _full(oracle, batch, layer), f"mid-mfma-{dtype}-{tile}", 2e-4, 2e-3)


@pytest.mark.parametrize("tile,bs,H", [(256, 8, 4), (320, 32, 3), (320, 4, 9), (256, 32, 1)])
def test_mfma_hidden_path_with_other_block_sizes_and_head_counts(oracle, tile, bs, H):
    """The MFMA kernel's gather through cache maps of 4-, 8- and 32-token blocks, with head counts that leave some of the
    eight head queues empty or uneven."""
    print(f"[case] mfma tile {tile} block_size {bs} heads {H}", flush=True)
    cfg = wl.small_config(name="mfmabs", dtype="f16", d_model=128 * H, n_heads=H, head_dim=128, block_size=bs,
                          batch=9, len_lo=1, len_hi=700, hidden_ratio=0.7)
    lens = np.array([700, 321, 1, 255, 33, 640, 31, 4, 97], dtype=np.int32)
    kinds = np.array([HID, HID, HID, KV, HID, HID, KV, HID, HID], dtype=np.uint8)
    batch = wl.make_batch(cfg, lens, kinds)
    layer = wl.make_layer(batch)
    rn, got = _run(batch, layer, hidden_chunk=tile)
    assert rn.info.hidden_impl == ab.APT_HIDDEN_MFMA and rn.info.hidden_chunk == tile
    _check(got, _full(oracle, batch, layer), f"mfma-{tile}-bs{bs}-H{H}", 2e-4, 2e-3)


@pytest.mark.parametrize("dtype,hd,H,bs", [("f32", 128, 2, 16), ("f16", 64, 4, 16), ("bf16", 64, 4, 8),
                                            ("f32", 64, 4, 4), ("f16", 128, 2, 32), ("f16", 128, 2, 4)])
def test_valu_hidden_and_kv_layout_variants(oracle, dtype, hd, H, bs):
    print(f"[case] valu {dtype} hd={hd} bs={bs}", flush=True)
    cfg = wl.small_config(name="var", dtype=dtype, d_model=hd * H, n_heads=H, head_dim=hd, block_size=bs,
                          batch=6, len_lo=1, len_hi=300, hidden_ratio=0.5)
    lens = np.array([300, 1, 65, 64, 17, 130], dtype=np.int32)
    kinds = np.array([KV, HID, HID, KV, KV, HID], dtype=np.uint8)
    batch = wl.make_batch(cfg, lens, kinds)
    layer = wl.make_layer(batch)
    rn, got = _run(batch, layer, hidden_impl=ab.APT_HIDDEN_VALU, kv_chunk=128)
    _check(got, _full(oracle, batch, layer), f"valu-{dtype}-hd{hd}-bs{bs}", 2e-4, 2e-3)


@pytest.mark.parametrize("dtype,hd,H,bs", [("f16", 128, 4, 16), ("bf16", 128, 4, 16), ("f32", 128, 2, 16),
                                            ("f16", 64, 6, 8), ("f32", 64, 5, 4)])
def test_absorbed_weight_hidden_path(oracle, dtype, hd, H, bs):
    # same step, hidden-kind requests through the re-associated form (no K/V projection)
    print(f"[case] absorbed {dtype} hd={hd} H={H} bs={bs}", flush=True)
    cfg = wl.small_config(name="absorbed", dtype=dtype, d_model=hd * H, n_heads=H, head_dim=hd, block_size=bs,
                          batch=8, len_lo=1, len_hi=1300, hidden_ratio=0.5)
    lens = np.array([1300, 257, 1, 512, 513, 256, 33, 1024], dtype=np.int32)
    kinds = np.array([HID, HID, HID, KV, KV, HID, KV, HID], dtype=np.uint8)
    batch = wl.make_batch(cfg, lens, kinds)
    layer = wl.make_layer(batch)
    rn, got = _run(batch, layer, hidden_impl=ab.APT_HIDDEN_ABSORBED)
    assert rn.info.hidden_impl == ab.APT_HIDDEN_ABSORBED
    _check(got, _full(oracle, batch, layer), f"absorbed-{dtype}-hd{hd}", 2e-4, 2e-3)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_absorbed_path_more_than_64_heads(oracle, dtype):
    # 66 heads: two groups of operand rows, the second with two heads only
    print(f"[case] absorbed 66 heads {dtype}", flush=True)
    cfg = wl.small_config(name="absorbed66", dtype=dtype, d_model=66 * 64, n_heads=66, head_dim=64, block_size=16,
                          batch=4, len_lo=1, len_hi=600, hidden_ratio=0.5)
    batch = wl.make_batch(cfg, np.array([70, 33, 530, 100], dtype=np.int32), np.array([HID, KV, HID, HID], dtype=np.uint8))
    layer = wl.make_layer(batch)
    _, got = _run(batch, layer, hidden_impl=ab.APT_HIDDEN_ABSORBED)
    _check(got, _full(oracle, batch, layer), f"absorbed-66-{dtype}", 2e-4, 2e-3)


def test_absorbed_path_requests_longer_than_2048_tokens(oracle):
    # more than 256 runs of 8 tokens per (request, head): the statistics kernel's second and third pass
    print("[case] absorbed long requests", flush=True)
    cfg = wl.small_config(name="absorbedlong", dtype="f16", d_model=256, n_heads=2, head_dim=128, block_size=16,
                          batch=3, len_lo=1, len_hi=4500, hidden_ratio=1.0)
    batch = wl.make_batch(cfg, np.array([4500, 2049, 10], dtype=np.int32), np.full(3, HID, dtype=np.uint8))
    layer = wl.make_layer(batch)
    _, got = _run(batch, layer, hidden_impl=ab.APT_HIDDEN_ABSORBED)
    _check(got, _full(oracle, batch, layer), "absorbed-long", 2e-4, 2e-3)


def test_absorbed_path_many_requests_pure_hidden_and_sixteen_bit_output(oracle):
    # more hidden-kind requests than one pass of the projection kernels holds (16), no KV-kind item
    print("[case] absorbed pure hidden, 19 requests", flush=True)
    cfg = wl.small_config(name="absorbed19", dtype="f16", d_model=512, n_heads=4, head_dim=128, block_size=16,
                          batch=19, len_lo=1, len_hi=600, hidden_ratio=1.0)
    batch = wl.make_batch(cfg)
    layer = wl.make_layer(batch)
    rn, got = _run(batch, layer, hidden_impl=ab.APT_HIDDEN_ABSORBED)
    _check(got, _full(oracle, batch, layer), "absorbed-19", 2e-4, 2e-3)
    _, got16 = _run(batch, layer, hidden_impl=ab.APT_HIDDEN_ABSORBED, out_dtype="f16")
    ref = torch.from_numpy(got.astype(np.float32)).to(torch.float16)
    assert np.array_equal(got16, ref.float().numpy().astype(np.float64))
    _, mf = _run(batch, layer)
    assert np.max(np.abs(got - mf)) < 1e-4


def test_mfma_and_valu_hidden_kernels_agree(oracle):
    print("[case] mfma vs valu", flush=True)
    cfg = wl.small_config(name="agree", dtype="f16", **{**MID, "batch": 3})
    batch = wl.make_batch(cfg, np.array([300, 40, 700], dtype=np.int32), np.full(3, HID, dtype=np.uint8))
    layer = wl.make_layer(batch)
    _, a = _run(batch, layer)
    _, b = _run(batch, layer, hidden_impl=ab.APT_HIDDEN_VALU)
    assert np.max(np.abs(a - b)) < 1e-4


@pytest.mark.parametrize("impl", [ab.APT_HIDDEN_AUTO, ab.APT_HIDDEN_ABSORBED])
def test_long_contexts_many_ranges_per_request(oracle, impl):
    # 16k-token requests: 64 hidden ranges / 32 KV ranges per (request, head) to merge
    print(f"[case] long contexts hidden_impl={impl}", flush=True)
    cfg = wl.small_config(name="long", dtype="bf16", d_model=256, n_heads=2, head_dim=128, block_size=16,
                          batch=4, len_lo=1, len_hi=16384, hidden_ratio=0.5)
    batch = wl.make_batch(cfg, np.array([16384, 16383, 9000, 5], dtype=np.int32), np.array([HID, KV, HID, KV], dtype=np.uint8))
    layer = wl.make_layer(batch)
    rn, got = _run(batch, layer, hidden_impl=impl)
    _check(got, _full(oracle, batch, layer), f"long-{impl}", 2e-4, 2e-3)


@pytest.mark.parametrize("kv_chunk,bs", [(1024, 16), (2048, 16), (2048, 8), (0, 16)])
def test_long_kv_ranges(oracle, kv_chunk, bs):
    """KV-kind ranges of 1024 and 2048 tokens (the lengths the planner picks by itself for large batches), with
    lengths around their boundaries, in a mixed batch and as the only kind (kv_chunk 0: 120 requests x 16 heads make the
    planner choose 1024 here); element by element against the oracle."""
    print(f"[case] long KV ranges kv_chunk={kv_chunk} block_size={bs}", flush=True)
    lens = [2048, 2047, 2049, 1024, 1025, 1023, 4096, 4097, 3000, 1, 700, 2050]
    kinds = [KV, KV, KV, KV, KV, KV, KV, KV, HID, KV, HID, KV]
    H = 4
    if kv_chunk == 0:
        g = np.random.default_rng(5)
        lens = [int(v) for v in g.integers(900, 1200, size=120)]
        kinds = [KV] * len(lens)
        H = 16
    cfg = wl.small_config(name="longkv", dtype="f16", d_model=128 * H, n_heads=H, head_dim=128, block_size=bs,
                          batch=len(lens), len_lo=1, len_hi=max(lens), hidden_ratio=0.5)
    batch = wl.make_batch(cfg, np.array(lens, dtype=np.int32), np.array(kinds, dtype=np.uint8))
    layer = wl.make_layer(batch)
    rn, got = _run(batch, layer, kv_chunk=kv_chunk)
    assert rn.info.kv_chunk == (kv_chunk or 1024)
    _check(got, _full(oracle, batch, layer), f"longkv-{kv_chunk}-{bs}")


@pytest.mark.parametrize("kinds", ["all_kv", "all_hidden"])
def test_pure_batches_and_single_request(oracle, kinds):
    print(f"[case] pure {kinds}", flush=True)
    cfg = wl.small_config(name="pure", dtype="f16", **{**MID, "batch": 4})
    k = np.full(4, KV if kinds == "all_kv" else HID, dtype=np.uint8)
    batch = wl.make_batch(cfg, np.array([1024, 511, 16, 15], dtype=np.int32), k)
    layer = wl.make_layer(batch)
    _, got = _run(batch, layer)
    _check(got, _full(oracle, batch, layer), f"pure-{kinds}", 2e-4, 2e-3)
    one = wl.make_batch(cfg, np.array([77], dtype=np.int32), k[:1])
    l1 = wl.make_layer(one)
    _, got = _run(one, l1)
    _check(got, _full(oracle, one, l1), f"single-{kinds}", 2e-4, 2e-3)


def test_page_permutation_is_bit_identical_on_gpu(oracle):
    print("[case] permuted pages", flush=True)
    seq = wl.small_config(name="perm", dtype="f16", poison=False, **MID)
    perm = replace(seq, permute_pages=True)
    bs_, bp_ = wl.make_batch(seq), wl.make_batch(perm)
    ls_, lp_ = wl.make_layer(bs_), wl.make_layer(bp_)
    for r in range(bs_.B):
        nb = (int(bs_.ctx_lens[r]) + 15) // 16
        for row in ((0, 1) if bs_.cache_kind[r] == KV else (0,)):
            for i in range(nb):
                lp_.pool[bp_.block_tables[r, row, i]] = ls_.pool[bs_.block_tables[r, row, i]]
    _, a = _run(bs_, ls_)
    _, b = _run(bp_, lp_)
    assert np.array_equal(a, b)
    _check(b, _full(oracle, bp_, lp_), "permuted", 2e-4, 2e-3)


def test_separate_pools_equal_unified_pool_and_poison_is_ignored(oracle):
    print("[case] pools + poison", flush=True)
    clean = wl.small_config(name="pois", dtype="f16", poison=False, **MID)
    dirty = replace(clean, poison=True)
    bc, bd = wl.make_batch(clean), wl.make_batch(dirty)
    lc, ld = wl.make_layer(bc), wl.make_layer(bd)
    _, a = _run(bc, lc)
    _, b = _run(bd, ld)
    _, c = _run(bd, ld, separate_pools=True)
    assert np.all(np.isfinite(b))
    assert np.array_equal(a, b) and np.array_equal(b, c)


def test_hidden_kind_equals_kv_kind_on_materialised_pages(oracle):
    # Section 3.1: K and V restored from the hidden cache are the K and V a KV cache would
    # hold.  Pages of the KV twin hold x W + b computed with numpy (float64, stored fp32).
    print("[case] hidden == kv", flush=True)
    cfg = wl.small_config(name="equiv", dtype="f32", d_model=256, n_heads=2, head_dim=128, block_size=16,
                          batch=3, len_lo=1, len_hi=200)
    lens = np.array([200, 31, 64], dtype=np.int32)
    bh = wl.make_batch(cfg, lens, np.full(3, HID, dtype=np.uint8))
    lh = wl.make_layer(bh)
    bk = wl.make_batch(cfg, lens, np.full(3, KV, dtype=np.uint8))
    lk = wl.make_layer(bk)
    lk.q[...] = lh.q
    W_K, W_V = lh.W_K.astype(np.float64), lh.W_V.astype(np.float64)
    for r in range(3):
        for j in range(int(lens[r])):
            x = wl.hidden_row_view(bh, lh.pool, r, j).astype(np.float64)
            wl.kv_row_view(bk, lk.pool, r, j, 0)[...] = (x @ W_K + lh.b_K).reshape(2, 128)
            wl.kv_row_view(bk, lk.pool, r, j, 1)[...] = (x @ W_V + lh.b_V).reshape(2, 128)
    _, a = _run(bh, lh)
    _, b = _run(bk, lk)
    assert np.max(np.abs(a - b)) < 5e-5


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_sixteen_bit_output(oracle, dtype):
    print(f"[case] out dtype {dtype}", flush=True)
    cfg = wl.small_config(name="odt", dtype=dtype, **{**MID, "batch": 3})
    batch = wl.make_batch(cfg, np.array([300, 40, 520], dtype=np.int32), np.array([HID, KV, KV], dtype=np.uint8))
    layer = wl.make_layer(batch)
    _, got32 = _run(batch, layer)
    _, got16 = _run(batch, layer, out_dtype=dtype)
    ref = torch.from_numpy(got32.astype(np.float32)).to(torch.float16 if dtype == "f16" else torch.bfloat16)
    assert np.array_equal(got16, ref.float().numpy().astype(np.float64))   # only the final rounding differs


def test_repeated_runs_are_bit_reproducible(oracle):
    print("[case] reproducible", flush=True)
    cfg = wl.small_config(name="repro", dtype="f16", **MID)
    batch = wl.make_batch(cfg)
    layer = wl.make_layer(batch)
    from paper_2504_07494_amd.harness import DecodeRunner
    rn = DecodeRunner(batch)
    dl = rn.upload(layer)
    rn.run(dl)
    first = rn.out_f64().copy()
    rn.workspace.fill_(0xFF)        # stale partials must not matter
    for _ in range(3):
        rn.plan()
        rn.run(dl)
        assert np.array_equal(rn.out_f64(), first)


def test_device_plan_copy_matches_host_plan(oracle):
    cfg = wl.small_config(name="plan", dtype="f16", **MID)
    batch = wl.make_batch(cfg)
    from paper_2504_07494_amd.harness import DecodeRunner
    rn = DecodeRunner(batch)
    torch.cuda.synchronize()
    n = int(rn.info.plan_bytes) // 4
    assert np.array_equal(rn.plan_dev[:n].cpu().numpy(), rn.plan_host[:n].numpy())


def test_steps_with_changing_lengths_back_to_back_without_a_device_sync(oracle):
    """A decode loop re-plans every step while earlier steps are still queued: each step's plan copy must reach
    the device intact (the host blob of a pending copy is never rewritten).  Five steps with different lengths
    and kinds are enqueued without any synchronisation; every step's output is then compared with the oracle."""
    print("[case] back-to-back re-planning", flush=True)
    from paper_2504_07494_amd.harness import DecodeRunner
    cfg = wl.small_config(name="replan", dtype="f16", d_model=1024, n_heads=8, head_dim=128, block_size=16, batch=24,
                          len_lo=600, len_hi=1500, hidden_ratio=0.5)
    batch = wl.make_batch(cfg)
    layer = wl.make_layer(batch)
    rn = DecodeRunner(batch)
    dl = rn.upload(layer)
    g = np.random.default_rng(7)
    steps = []
    for i in range(5):
        lens = np.maximum(1, (batch.ctx_lens * g.uniform(0.05, 1.0, size=batch.B)).astype(np.int32))
        if i == 4:
            lens = batch.ctx_lens.copy()
        steps.append((lens, batch.cache_kind.copy()))
    outs = [torch.empty_like(rn.out) for _ in steps]
    torch.cuda.synchronize()
    for (lens, kinds), out in zip(steps, outs):      # no synchronisation inside this loop
        rn.plan(lens, kinds)
        rn.run(dl, out=out)
    torch.cuda.synchronize()
    c = batch.cfg
    for i, ((lens, kinds), out) in enumerate(zip(steps, outs)):
        want = oracle.attn(oracle.shape_of(c.d_model, c.n_heads, c.head_dim, c.block_size, c.dtype, batch.max_blocks,
                                           c.softmax_scale), layer.q, layer.pool, layer.pool, layer.pool, layer.W_K,
                           layer.b_K, layer.W_V, layer.b_V, batch.block_tables, lens, kinds).reshape(out.shape)
        _check(out.float().cpu().numpy().astype(np.float64), want, f"replan step {i}")
