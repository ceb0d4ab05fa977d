"""Cache append (the step before the attention path): oracle pins on the CPU, bit-exact
GPU parity through the C ABI."""
import os

import numpy as np
import pytest

from oracle import plan_oracle as po
from paper_2504_07494_amd import workloads as wl
from tests.helpers import oracle_attn, oracle_shape
from tests.test_oracle_pins import _read_pool_example

KV, HID = wl.KIND_KV, wl.KIND_HIDDEN


def _new_vectors(cfg, B, seed):
    g = np.random.default_rng(seed)
    x = wl.round_to_dtype(g.standard_normal((B, cfg.d_model), dtype=np.float32), cfg.dtype)
    k = wl.round_to_dtype(g.standard_normal((B, cfg.n_heads, cfg.head_dim), dtype=np.float32), cfg.dtype)
    v = wl.round_to_dtype(g.standard_normal((B, cfg.n_heads, cfg.head_dim), dtype=np.float32), cfg.dtype)
    return x, k, v


def test_oracle_append_writes_the_paper_example_positions(oracle):
    # Section 4.3 example: A (KV, 11 tokens) -> token 10 = K block 4 / V block 12, slot 2;
    # B (hidden, 14 tokens) -> token 13 = block 15, slot 1
    ex = _read_pool_example()
    bs, d, H, hd = ex["block_size"], 8, 2, 4
    bt = np.full((2, 2, 4), -1, dtype=np.int32)
    bt[0, 0, :3] = ex["A"]["k_blocks"]; bt[0, 1, :3] = ex["A"]["v_blocks"]; bt[1, 0, :4] = ex["B"]["h_blocks"]
    ctx = np.array([11, 14], dtype=np.int32)
    kinds = np.array([KV, HID], dtype=np.uint8)
    pool = np.zeros((ex["pool_blocks"], bs * d), dtype=np.float32)
    x = np.arange(2 * d, dtype=np.float32).reshape(2, d) + 100
    k = np.arange(2 * d, dtype=np.float32).reshape(2, H, hd) + 200
    v = np.arange(2 * d, dtype=np.float32).reshape(2, H, hd) + 300
    sh = oracle.shape_of(d, H, hd, bs, "f32", 4, 1.0)
    oracle.append(sh, x, k, v, pool, pool, pool, bt, ctx, kinds)
    want = np.zeros_like(pool)
    want[4].reshape(H, bs, hd)[:, 2, :] = k[0]
    want[12].reshape(H, bs, hd)[:, 2, :] = v[0]
    want[15].reshape(bs, d)[1, :] = x[1]
    assert np.array_equal(pool, want)
    assert po.token_location(ex["A"]["k_blocks"], bs, 10) == (4, 2)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_oracle_append_then_attention_sees_the_new_token(oracle, dtype):
    # after the append the attention over n tokens must equal the attention computed with the
    # vectors placed through the layout accessors of the input generator (independent index code)
    cfg = wl.small_config(batch=5, len_hi=37, dtype=dtype, poison=False)
    b = wl.make_batch(cfg)
    l = wl.make_layer(b)
    x, k, v = _new_vectors(cfg, b.B, 3)
    ref_pool = l.pool.copy()
    for r in range(b.B):
        j = int(b.ctx_lens[r]) - 1
        if b.cache_kind[r] == HID:
            wl.hidden_row_view(b, ref_pool, r, j)[...] = x[r]
        else:
            wl.kv_row_view(b, ref_pool, r, j, 0)[...] = k[r]
            wl.kv_row_view(b, ref_pool, r, j, 1)[...] = v[r]
    got_pool = l.pool.copy()
    oracle.append(oracle_shape(oracle, b), x, k, v, got_pool, got_pool, got_pool, b.block_tables, b.ctx_lens, b.cache_kind)
    assert np.array_equal(got_pool.view(np.uint8), ref_pool.view(np.uint8))
    assert not np.array_equal(got_pool.view(np.uint8), l.pool.view(np.uint8))
    # n = 1: the output is the appended value itself
    one = wl.make_batch(cfg, np.ones(2, dtype=np.int32), np.array([KV, KV], dtype=np.uint8))
    l1 = wl.make_layer(one)
    x1, k1, v1 = _new_vectors(cfg, 2, 4)
    oracle.append(oracle_shape(oracle, one), x1, k1, v1, l1.pool, l1.pool, l1.pool, one.block_tables, one.ctx_lens, one.cache_kind)
    out = oracle_attn(oracle, one, l1).reshape(2, cfg.n_heads, cfg.head_dim)
    assert np.array_equal(out, wl.to_f64(v1, dtype))


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,hd,H,bs", [("f16", 128, 4, 16), ("f32", 64, 4, 16), ("bf16", 128, 2, 4)])
def test_gpu_append_is_bit_exact_and_feeds_the_attention(oracle, dtype, hd, H, bs):
    import torch
    from paper_2504_07494_amd import binding as ab
    from paper_2504_07494_amd.harness import DecodeRunner, _to_dev
    print(f"[case] append {dtype} hd={hd} bs={bs}", flush=True)
    cfg = wl.small_config(name="app", dtype=dtype, d_model=hd * H, n_heads=H, head_dim=hd, block_size=bs,
                          batch=9, len_lo=1, len_hi=300, hidden_ratio=0.5, poison=False)
    batch = wl.make_batch(cfg)
    layer = wl.make_layer(batch)
    x, k, v = _new_vectors(cfg, batch.B, 5)
    want_pool = layer.pool.copy()
    oracle.append(oracle_shape(oracle, batch), x, k, v, want_pool, want_pool, want_pool, batch.block_tables,
                  batch.ctx_lens, batch.cache_kind)
    rn = DecodeRunner(batch)
    dl = rn.upload(layer)
    ab.apt_cache_append(rn.shape, batch.B, _to_dev(x, rn.device), _to_dev(k, rn.device), _to_dev(v, rn.device),
                        dl.pool, dl.pool, dl.pool, rn.block_tables,
                        torch.from_numpy(batch.ctx_lens).to(rn.device), torch.from_numpy(batch.cache_kind).to(rn.device),
                        rn.stream())
    torch.cuda.synchronize()
    got_pool = dl.pool.cpu().numpy()
    assert np.array_equal(got_pool.view(np.uint8).reshape(-1), want_pool.view(np.uint8).reshape(-1))
    # and the attention over the appended cache matches the oracle on the oracle-appended pool
    rn.run(dl)
    got = rn.out_f64()
    layer.pool[...] = want_pool
    want = oracle_attn(oracle, batch, layer).reshape(got.shape)
    assert np.max(np.abs(got - want)) < 2e-4
