"""Host-side checks of the seeded input generator (no method arithmetic in it)."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from paper_2504_07494_amd import workloads as wl


def test_bf16_rounding_matches_torch():
    g = np.random.default_rng(0)
    a = np.concatenate([g.standard_normal(5000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40], dtype=np.float32)])
    bits = wl.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    back = wl.bf16_bits_to_f32(bits)
    assert np.array_equal(back, torch.from_numpy(a).to(torch.bfloat16).float().numpy())


def test_generation_is_deterministic_and_thread_independent():
    cfg = wl.small_config(batch=6, len_hi=60, d_model=128, n_heads=4, head_dim=32)
    b1, b2 = wl.make_batch(cfg), wl.make_batch(cfg)
    l1, l2 = wl.make_layer(b1, workers=1), wl.make_layer(b2, workers=4)
    for name in ("pool", "W_K", "W_V", "b_K", "b_V", "q"):
        assert np.array_equal(getattr(l1, name), getattr(l2, name), equal_nan=True)
    l3 = wl.make_layer(b1, layer=1)
    assert not np.array_equal(l1.W_K, l3.W_K)


@pytest.mark.parametrize("name", ["tiny", "opt13b", "opt30b", "opt66b", "opt13b_step"])
def test_config_metadata(name):
    cfg = wl.CONFIGS[name]
    b = wl.make_batch(cfg)
    assert cfg.n_heads * cfg.head_dim == cfg.d_model
    assert b.B == cfg.batch
    assert b.ctx_lens.min() >= cfg.len_lo and b.ctx_lens.max() <= cfg.len_hi
    # every referenced block id is unique and inside the pool
    nb = (b.ctx_lens.astype(np.int64) + cfg.block_size - 1) // cfg.block_size
    used = []
    for r in range(b.B):
        used.extend(b.block_tables[r, 0, :nb[r]])
        assert np.all(b.block_tables[r, 0, nb[r]:] == -1)
        if b.cache_kind[r] == wl.KIND_KV:
            used.extend(b.block_tables[r, 1, :nb[r]])
        else:
            assert np.all(b.block_tables[r, 1] == -1)
    used = np.array(used)
    assert len(np.unique(used)) == len(used)
    assert used.min() >= 0 and used.max() < b.n_pool_blocks
    if cfg.kind_rule == "ratio":
        assert int((b.cache_kind == wl.KIND_HIDDEN).sum()) == int(np.floor(cfg.hidden_ratio * cfg.batch + 0.5))
    if cfg.permute_pages:
        assert not np.all(np.diff(b.block_tables[0, 0, :nb[0]]) == 1)


def test_ratio_sweep_sets_are_nested():
    cfg = wl.CONFIGS["opt66b"]
    prev = np.zeros(cfg.batch, dtype=bool)
    lens0 = wl.draw_ctx_lens(cfg)
    for ratio, count in [(0.0, 0), (0.25, 64), (0.5, 128), (0.75, 192), (1.0, 256)]:
        c = wl.with_ratio(cfg, ratio)
        kind = wl.draw_cache_kind(c) == wl.KIND_HIDDEN
        assert kind.sum() == count
        assert np.all(kind[prev])
        assert np.array_equal(wl.draw_ctx_lens(c), lens0)
        prev = kind


def test_value_distributions():
    cfg = replace(wl.CONFIGS["tiny"], batch=16, len_hi=128, poison=False)
    b = wl.make_batch(cfg)
    l = wl.make_layer(b)
    assert abs(float(l.W_K.std()) - 0.02) < 2e-3 and abs(float(l.q.std()) - 1.0) < 0.1
    hid = l.pool[b.block_type == 3]
    kv = l.pool[(b.block_type == 1) | (b.block_type == 2)]
    assert abs(float(hid.std()) - 1.0) < 0.05
    assert abs(float(kv.std()) - cfg.kv_std) / cfg.kv_std < 0.05


def test_poison_marks_only_unused_slots():
    cfg = wl.small_config(batch=5, len_hi=30, poison=True)
    b = wl.make_batch(cfg)
    l = wl.make_layer(b)
    for r in range(b.B):
        for j in range(int(b.ctx_lens[r])):
            if b.cache_kind[r] == wl.KIND_HIDDEN:
                assert not np.isnan(wl.hidden_row_view(b, l.pool, r, j)).any()
            else:
                assert not np.isnan(wl.kv_row_view(b, l.pool, r, j, 0)).any()
                assert not np.isnan(wl.kv_row_view(b, l.pool, r, j, 1)).any()
    assert np.isnan(l.pool[b.block_type == 0]).all()
