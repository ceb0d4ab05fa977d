"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU library.  Each pin is chosen so that a
plausible mistake in the oracle (dropped bias, wrong sign, transposed weight,
wrong head slice, wrong block/slot arithmetic, missing normalisation) fails it.
"""
import math
import os
from dataclasses import replace

import numpy as np
import pytest

from paper_2504_07494_amd import workloads as wl
from tests.helpers import brute_force_attention, logical_kv, oracle_attn, oracle_shape

KV, HID = wl.KIND_KV, wl.KIND_HIDDEN


def _cfg(**kw):
    return wl.small_config(**kw)


def _materialise_as_kv(batch_h, layer_h, exact_f64=True):
    """KV-kind twin of an all-hidden batch: pages hold K = X W + b, V = X W + b
    computed with numpy in float64 and stored in the config dtype."""
    cfg = batch_h.cfg
    kinds = np.full(batch_h.B, KV, dtype=np.uint8)
    batch_k = wl.make_batch(cfg, batch_h.ctx_lens, kinds)
    layer_k = wl.make_layer(batch_k)
    for r in range(batch_h.B):
        K, V = logical_kv(batch_h, layer_h, r)
        for j in range(int(batch_h.ctx_lens[r])):
            wl.kv_row_view(batch_k, layer_k.pool, r, j, 0)[...] = wl.round_to_dtype(K[j].astype(np.float32), cfg.dtype)
            wl.kv_row_view(batch_k, layer_k.pool, r, j, 1)[...] = wl.round_to_dtype(V[j].astype(np.float32), cfg.dtype)
    layer_k.q[...] = layer_h.q
    return batch_k, layer_k


# --- P1: hidden kind == KV kind on materialised x W + b (Section 3.1) --------------
def test_hidden_equals_kv_random(oracle):
    cfg = _cfg(batch=4, len_hi=37)
    bh = wl.make_batch(cfg, cache_kind=np.full(4, HID, dtype=np.uint8))
    lh = wl.make_layer(bh)
    bk, lk = _materialise_as_kv(bh, lh)
    oh = oracle_attn(oracle, bh, lh)
    ok = oracle_attn(oracle, bk, lk)
    # pages are fp32: the materialised K/V carry one fp32 rounding each
    assert np.max(np.abs(oh - ok)) < 2e-6
    assert np.max(np.abs(oh)) > 0.05


def test_hidden_equals_kv_exact_integers(oracle):
    # integer-valued x, dyadic W and b: x W + b is exact in fp32, so both kinds
    # must agree to double rounding
    cfg = _cfg(batch=3, len_hi=21, d_model=32, n_heads=4, head_dim=8)
    bh = wl.make_batch(cfg, cache_kind=np.full(3, HID, dtype=np.uint8))
    lh = wl.make_layer(bh)
    g = np.random.default_rng(5)
    valid = ~np.isnan(lh.pool)
    lh.pool[valid] = g.integers(-3, 4, size=int(valid.sum())).astype(np.float32)
    lh.W_K[...] = g.integers(-4, 5, size=lh.W_K.shape) / 8.0
    lh.W_V[...] = g.integers(-4, 5, size=lh.W_V.shape) / 8.0
    lh.b_K[...] = g.integers(-4, 5, size=lh.b_K.shape) / 4.0
    lh.b_V[...] = g.integers(-4, 5, size=lh.b_V.shape) / 4.0
    lh.q[...] = g.integers(-2, 3, size=lh.q.shape) / 4.0
    bk, lk = _materialise_as_kv(bh, lh)
    oh = oracle_attn(oracle, bh, lh)
    ok = oracle_attn(oracle, bk, lk)
    assert np.max(np.abs(oh - ok)) < 1e-12
    assert np.max(np.abs(oh)) > 0.1


# --- P2: softmax weights are a probability vector (Eq. 2) ---------------------------
def test_softmax_weights_sum_to_one(oracle):
    cfg = _cfg(batch=5, len_hi=50)
    b = wl.make_batch(cfg)
    l = wl.make_layer(b)
    out, w = oracle_attn(oracle, b, l, want_weights=True)
    assert len(w) == b.B * cfg.n_heads
    for p, a in enumerate(w):
        assert len(a) == b.ctx_lens[p // cfg.n_heads]
        assert np.all(a >= 0.0)
        assert abs(a.sum() - 1.0) < 1e-12


# --- P3: brute force on tiny inputs, incl. the 3-token, dimension-3 shape of the
# KV-vs-hidden-cache figure (Section 3.1) -----------------------------------------------
@pytest.mark.parametrize("d,H,hd,bs,lens", [(3, 1, 3, 2, [3, 3]), (8, 2, 4, 4, [1, 5, 8, 7]), (6, 3, 2, 16, [8, 2])])
def test_brute_force_tiny(oracle, d, H, hd, bs, lens):
    cfg = _cfg(d_model=d, n_heads=H, head_dim=hd, block_size=bs, batch=len(lens), len_hi=max(lens), w_std=0.4)
    kinds = np.array([HID if i % 2 == 0 else KV for i in range(len(lens))], dtype=np.uint8)
    b = wl.make_batch(cfg, np.array(lens, dtype=np.int32), kinds)
    l = wl.make_layer(b)
    out = oracle_attn(oracle, b, l).reshape(b.B, H, hd)
    qs = wl.to_f64(l.q, cfg.dtype)
    for r in range(b.B):
        K, V = logical_kv(b, l, r)
        for h in range(H):
            ref = brute_force_attention(qs[r, h], K[:, h, :], V[:, h, :], cfg.softmax_scale)
            assert np.max(np.abs(out[r, h] - ref)) < 1e-12


# --- P4: closed forms ---------------------------------------------------------------
def test_single_token_returns_its_value(oracle):
    cfg = _cfg(batch=2, len_lo=1, len_hi=1)
    b = wl.make_batch(cfg, np.array([1, 1], dtype=np.int32), np.array([HID, KV], dtype=np.uint8))
    l = wl.make_layer(b)
    out = oracle_attn(oracle, b, l).reshape(2, cfg.n_heads, cfg.head_dim)
    for r in range(2):
        _, V = logical_kv(b, l, r)
        assert np.max(np.abs(out[r] - V[0])) < 1e-13


def test_zero_query_gives_mean_value(oracle):
    cfg = _cfg(batch=4, len_hi=33)
    b = wl.make_batch(cfg)
    l = wl.make_layer(b)
    l.q[...] = 0
    out = oracle_attn(oracle, b, l).reshape(b.B, cfg.n_heads, cfg.head_dim)
    for r in range(b.B):
        _, V = logical_kv(b, l, r)
        assert np.max(np.abs(out[r] - V.mean(axis=0))) < 1e-12


def test_zero_key_weights_give_mean_value(oracle):
    cfg = _cfg(batch=2, len_hi=19)
    b = wl.make_batch(cfg, cache_kind=np.full(2, HID, dtype=np.uint8))
    l = wl.make_layer(b)
    l.W_K[...] = 0
    out = oracle_attn(oracle, b, l).reshape(b.B, cfg.n_heads, cfg.head_dim)
    for r in range(b.B):
        _, V = logical_kv(b, l, r)          # b_K stays non-zero: a constant shift of all scores
        assert np.max(np.abs(out[r] - V.mean(axis=0))) < 1e-12


def test_equal_tokens_return_the_common_value(oracle):
    cfg = _cfg(batch=1, len_hi=11, block_size=4)
    b = wl.make_batch(cfg, np.array([11], dtype=np.int32), np.array([HID], dtype=np.uint8))
    l = wl.make_layer(b)
    x0 = wl.hidden_row_view(b, l.pool, 0, 0).copy()
    for j in range(11):
        wl.hidden_row_view(b, l.pool, 0, j)[...] = x0
    out = oracle_attn(oracle, b, l).reshape(cfg.n_heads, cfg.head_dim)
    _, V = logical_kv(b, l, 0)
    assert np.max(np.abs(out - V[0])) < 1e-12


def test_identity_weights_reduce_to_attention_over_x(oracle):
    # W_K = W_V = I, b = 0: the hidden kind must equal the KV kind whose K and V pages
    # both hold x (head h sees channels h*hd..(h+1)*hd of x)
    cfg = _cfg(batch=2, len_hi=23)
    bh = wl.make_batch(cfg, cache_kind=np.full(2, HID, dtype=np.uint8))
    lh = wl.make_layer(bh)
    lh.W_K[...] = np.eye(cfg.d_model, dtype=np.float32)
    lh.W_V[...] = np.eye(cfg.d_model, dtype=np.float32)
    lh.b_K[...] = 0
    lh.b_V[...] = 0
    bk = wl.make_batch(cfg, bh.ctx_lens, np.full(2, KV, dtype=np.uint8))
    lk = wl.make_layer(bk)
    lk.q[...] = lh.q
    for r in range(2):
        for j in range(int(bh.ctx_lens[r])):
            x = wl.hidden_row_view(bh, lh.pool, r, j).reshape(cfg.n_heads, cfg.head_dim)
            wl.kv_row_view(bk, lk.pool, r, j, 0)[...] = x
            wl.kv_row_view(bk, lk.pool, r, j, 1)[...] = x
    assert np.max(np.abs(oracle_attn(oracle, bh, lh) - oracle_attn(oracle, bk, lk))) < 1e-13


def test_zero_bias_reduces_to_eq1(oracle):
    # with b = 0 the projection is exactly Eq. 1 (k = W x): compare with numpy
    cfg = _cfg(batch=2, len_hi=9)
    b = wl.make_batch(cfg, cache_kind=np.full(2, HID, dtype=np.uint8))
    l = wl.make_layer(b)
    out_b = oracle_attn(oracle, b, l)
    l.b_K[...] = 0
    l.b_V[...] = 0
    out_0 = oracle_attn(oracle, b, l).reshape(b.B, cfg.n_heads, cfg.head_dim)
    assert np.max(np.abs(out_b.reshape(out_0.shape) - out_0)) > 1e-4      # the bias is really used
    qs = wl.to_f64(l.q, cfg.dtype)
    for r in range(b.B):
        K, V = logical_kv(b, l, r)
        for h in range(cfg.n_heads):
            ref = brute_force_attention(qs[r, h], K[:, h], V[:, h], cfg.softmax_scale)
            assert np.max(np.abs(out_0[r, h] - ref)) < 1e-12


def test_scale_is_applied_to_scores(oracle):
    # scale -> 0 gives the mean; a different scale changes the result; 1/sqrt(head_dim)
    # is what the workloads pass
    cfg = _cfg(batch=2, len_hi=17)
    b = wl.make_batch(cfg)
    l = wl.make_layer(b)
    assert abs(cfg.softmax_scale - 1.0 / math.sqrt(cfg.head_dim)) < 1e-15
    o0 = oracle_attn(oracle, b, l, scale=0.0).reshape(b.B, cfg.n_heads, cfg.head_dim)
    for r in range(b.B):
        _, V = logical_kv(b, l, r)
        assert np.max(np.abs(o0[r] - V.mean(axis=0))) < 1e-12
    qs = wl.to_f64(l.q, cfg.dtype)
    o2 = oracle_attn(oracle, b, l, scale=0.7).reshape(b.B, cfg.n_heads, cfg.head_dim)
    K, V = logical_kv(b, l, 1)
    ref = brute_force_attention(qs[1, 0], K[:, 0], V[:, 0], 0.7)
    assert np.max(np.abs(o2[1, 0] - ref)) < 1e-12


# --- P5: absorbed-weight identity (second derivation of Eq. 1-3) ----------------------
def test_absorbed_weight_identity(oracle):
    cfg = _cfg(batch=3, len_hi=29, d_model=48, n_heads=3, head_dim=16)
    b = wl.make_batch(cfg, cache_kind=np.full(3, HID, dtype=np.uint8))
    l = wl.make_layer(b)
    out = oracle_attn(oracle, b, l).reshape(b.B, cfg.n_heads, cfg.head_dim)
    WK, WV = wl.to_f64(l.W_K, cfg.dtype), wl.to_f64(l.W_V, cfg.dtype)
    bK, bV = wl.to_f64(l.b_K, cfg.dtype), wl.to_f64(l.b_V, cfg.dtype)
    qs = wl.to_f64(l.q, cfg.dtype)
    hd = cfg.head_dim
    for r in range(b.B):
        n = int(b.ctx_lens[r])
        X = np.stack([wl.to_f64(wl.hidden_row_view(b, l.pool, r, j), cfg.dtype) for j in range(n)])
        for h in range(cfg.n_heads):
            sl = slice(h * hd, (h + 1) * hd)
            qt = WK[:, sl] @ qs[r, h]                       # absorbed query, length d
            s = cfg.softmax_scale * (X @ qt + qs[r, h] @ bK[sl])
            a = np.exp(s - s.max())
            a /= a.sum()
            ref = (a @ X) @ WV[:, sl] + bV[sl]              # uses sum(a) = 1
            assert np.max(np.abs(out[r, h] - ref)) < 1e-11


# --- P6: split invariance of partial + merge --------------------------------------------
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_split_invariance(oracle, seed):
    cfg = _cfg(batch=2, len_lo=20, len_hi=45, block_size=4)
    b = wl.make_batch(cfg, cache_kind=np.array([HID, KV], dtype=np.uint8))
    l = wl.make_layer(b)
    full = oracle_attn(oracle, b, l).reshape(b.B, cfg.n_heads, cfg.head_dim)
    sh = oracle_shape(oracle, b)
    g = np.random.default_rng(seed)
    for r in range(b.B):
        n = int(b.ctx_lens[r])
        if seed == 0:
            cuts = list(range(n + 1))                      # one-token ranges
        else:
            inner = np.sort(g.choice(np.arange(1, n), size=g.integers(1, 6), replace=False))
            cuts = [0] + [int(c) for c in inner] + [n]     # arbitrary, cutting inside blocks
        for h in range(cfg.n_heads):
            ms, ls, accs = [], [], []
            for t0, t1 in zip(cuts[:-1], cuts[1:]):
                m, lsum, acc = oracle.partial(sh, l.q, l.pool, l.pool, l.pool, l.W_K, l.b_K, l.W_V, l.b_V,
                                              b.block_tables, b.cache_kind[r], r, h, t0, t1)
                ms.append(m); ls.append(lsum); accs.append(acc)
            merged = oracle.merge(ms, ls, np.stack(accs))
            assert np.max(np.abs(merged - full[r, h])) < 1e-12


def test_merge_of_one_partial_normalises(oracle):
    out = oracle.merge([3.0], [4.0], np.array([[2.0, 8.0]]))
    assert np.allclose(out, [0.5, 2.0], rtol=0, atol=1e-15)
    # two partials with different maxima: hand-computed
    m = [0.0, math.log(2.0)]
    out = oracle.merge(m, [1.0, 1.0], np.array([[1.0], [3.0]]))
    # weights exp(m - m*) = 1/2 and 1: (0.5*1 + 3) / (0.5 + 1)
    assert abs(out[0] - 3.5 / 1.5) < 1e-15


# --- P7: physical placement does not matter (Section 4.3) -------------------------------
def test_page_permutation_is_bit_identical(oracle):
    cfg_seq = _cfg(batch=4, len_hi=40, permute_pages=False, poison=False)
    cfg_perm = replace(cfg_seq, permute_pages=True)
    bs_, bp_ = wl.make_batch(cfg_seq), wl.make_batch(cfg_perm)
    assert np.array_equal(bs_.ctx_lens, bp_.ctx_lens) and np.array_equal(bs_.cache_kind, bp_.cache_kind)
    ls_ = wl.make_layer(bs_)
    lp_ = wl.make_layer(bp_)
    # move the sequential pool's logical content to the permuted placement
    for r in range(bs_.B):
        nb = (int(bs_.ctx_lens[r]) + cfg_seq.block_size - 1) // cfg_seq.block_size
        rows = (0, 1) if bs_.cache_kind[r] == KV else (0,)
        for row in rows:
            for i in range(nb):
                lp_.pool[bp_.block_tables[r, row, i]] = ls_.pool[bs_.block_tables[r, row, i]]
    for name in ("W_K", "W_V", "b_K", "b_V", "q"):
        assert np.array_equal(getattr(ls_, name), getattr(lp_, name))
    assert not np.array_equal(bs_.block_tables, bp_.block_tables)
    o1 = oracle_attn(oracle, bs_, ls_)
    o2 = oracle_attn(oracle, bp_, lp_)
    assert np.array_equal(o1, o2)


def test_separate_pools_equal_unified_pool(oracle):
    # K, V and hidden blocks may live in one pool or in three (Section 4.3)
    cfg = _cfg(batch=4, len_hi=30)
    b = wl.make_batch(cfg)
    l = wl.make_layer(b)
    o1 = oracle_attn(oracle, b, l)
    kp, vp, hp = l.pool.copy(), l.pool.copy(), l.pool.copy()
    kp[b.block_type != 1] = np.nan
    vp[b.block_type != 2] = np.nan
    hp[b.block_type != 3] = np.nan
    o2 = oracle.attn(oracle_shape(oracle, b), l.q, kp, vp, hp, l.W_K, l.b_K, l.W_V, l.b_V,
                     b.block_tables, b.ctx_lens, b.cache_kind)
    assert np.array_equal(o1, o2)


# --- P8: the paper's worked block mapping (Section 4.3) --------------------------------
def _read_pool_example():
    path = os.path.join(os.path.dirname(__file__), "golden", "pool_example.txt")
    ex = {}
    for line in open(path):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] in ("pool_blocks", "block_size"):
            ex[t[0]] = int(t[1])
        else:
            rec = {"kind": t[2], "tokens": int(t[4])}
            key = None
            for tok in t[5:]:
                if tok.endswith("_blocks"):
                    key = tok
                    rec[key] = []
                else:
                    rec[key].append(int(tok))
            ex[t[0]] = rec
    return ex


def test_paper_pool_example_indexing(oracle):
    from oracle import plan_oracle as po
    ex = _read_pool_example()
    bs = ex["block_size"]
    A, Bq = ex["A"], ex["B"]
    assert po.blocks_for(A["tokens"], bs) == len(A["k_blocks"]) == len(A["v_blocks"]) == 3
    assert po.blocks_for(Bq["tokens"], bs) == len(Bq["h_blocks"]) == 4
    assert po.token_location(A["k_blocks"], bs, 10) == (4, 2)
    assert po.token_location(A["v_blocks"], bs, 10) == (12, 2)
    assert po.token_location(Bq["h_blocks"], bs, 13) == (15, 1)
    assert po.token_location(Bq["h_blocks"], bs, 4) == (7, 0)

    # the same mapping through the C oracle: one-hot attention on marker values
    d, H, hd = 8, 2, 4
    cfg = _cfg(d_model=d, n_heads=H, head_dim=hd, block_size=bs, batch=2, len_hi=16, poison=False)
    bt = np.full((2, 2, 4), -1, dtype=np.int32)
    bt[0, 0, :3] = A["k_blocks"]; bt[0, 1, :3] = A["v_blocks"]; bt[1, 0, :4] = Bq["h_blocks"]
    ctx = np.array([A["tokens"], Bq["tokens"]], dtype=np.int32)
    kinds = np.array([KV, HID], dtype=np.uint8)
    pool = np.zeros((ex["pool_blocks"], bs * d), dtype=np.float32)
    sh = oracle.shape_of(d, H, hd, bs, "f32", 4, 1.0)
    q = np.zeros((2, H, hd), dtype=np.float32)
    q[:, :, 0] = 1.0
    # request A: V rows carry the marker 100*block + 10*slot + head; token j* gets a huge key
    for blk in A["v_blocks"]:
        v = pool[blk].reshape(H, bs, hd)
        for h in range(H):
            for s in range(bs):
                v[h, s, :] = 100 * blk + 10 * s + h
    W0 = np.zeros((d, d), dtype=np.float32)
    b0 = np.zeros(d, dtype=np.float32)
    for jstar in (0, 5, 10):
        kp = pool.copy()
        blk, slot = po.token_location(A["k_blocks"], bs, jstar)
        kp[blk].reshape(H, bs, hd)[:, slot, 0] = 80.0
        out = oracle.attn(sh, q, kp, kp, kp, W0, b0, W0, b0, bt, ctx, kinds, pairs=[(0, 0), (0, 1)])
        vb, vs = po.token_location(A["v_blocks"], bs, jstar)
        assert np.allclose(out[0], 100 * vb + 10 * vs + 0, atol=1e-9)
        assert np.allclose(out[1], 100 * vb + 10 * vs + 1, atol=1e-9)
    # request B: x rows carry markers; W_K picks channel 0 into every head's channel 0,
    # W_V copies channel 1 of x to all outputs
    WK = np.zeros((d, d), dtype=np.float32); WK[0, 0] = 1.0; WK[0, hd] = 1.0
    WV = np.zeros((d, d), dtype=np.float32); WV[1, :] = 1.0
    for jstar in (4, 13):
        hp = np.zeros_like(pool)
        for blk in Bq["h_blocks"]:
            x = hp[blk].reshape(bs, d)
            for s in range(bs):
                x[s, 1] = 100 * blk + 10 * s
        blk, slot = po.token_location(Bq["h_blocks"], bs, jstar)
        hp[blk].reshape(bs, d)[slot, 0] = 80.0
        out = oracle.attn(sh, q, hp, hp, hp, WK, b0, WV, b0, bt, ctx, kinds, pairs=[(1, 0), (1, 1)])
        assert np.allclose(out, 100 * blk + 10 * slot, atol=1e-9)


# --- P9: the hidden cache needs half the storage of the KV cache (Section 3.1) ---------
def test_hidden_cache_is_half_the_kv_cache():
    from oracle import plan_oracle as po
    for n in (1, 11, 14, 2048):
        assert 2 * po.cache_bytes(n, 5120, 2, HID) == po.cache_bytes(n, 5120, 2, KV)
    cfg = _cfg(batch=6, len_hi=40)
    lens = wl.draw_ctx_lens(cfg)
    all_h = wl.make_batch(cfg, lens, np.full(6, HID, dtype=np.uint8))
    all_k = wl.make_batch(cfg, lens, np.full(6, KV, dtype=np.uint8))
    assert 2 * int((all_h.block_type == 3).sum()) == int((all_k.block_type > 0).sum())


# --- P10: no positional term; masked slots are never read ------------------------------
def test_token_order_permutation_invariance(oracle):
    cfg = _cfg(batch=2, len_hi=26, poison=False)
    b = wl.make_batch(cfg, cache_kind=np.array([HID, KV], dtype=np.uint8))
    l = wl.make_layer(b)
    o1 = oracle_attn(oracle, b, l)
    g = np.random.default_rng(3)
    pool2 = l.pool.copy()
    for r in range(2):
        n = int(b.ctx_lens[r])
        perm = g.permutation(n)
        if b.cache_kind[r] == HID:
            rows = [wl.hidden_row_view(b, l.pool, r, j).copy() for j in range(n)]
            for j in range(n):
                wl.hidden_row_view(b, pool2, r, j)[...] = rows[perm[j]]
        else:
            for which in (0, 1):
                rows = [wl.kv_row_view(b, l.pool, r, j, which).copy() for j in range(n)]
                for j in range(n):
                    wl.kv_row_view(b, pool2, r, j, which)[...] = rows[perm[j]]
    l2 = replace(l, pool=pool2)
    o2 = oracle_attn(oracle, b, l2)
    assert np.max(np.abs(o1 - o2)) < 1e-12


def test_poison_in_unused_slots_is_never_read(oracle):
    clean = _cfg(batch=5, len_hi=39, poison=False)
    dirty = replace(clean, poison=True)
    bc, bd = wl.make_batch(clean), wl.make_batch(dirty)
    lc, ld = wl.make_layer(bc), wl.make_layer(bd)
    assert np.isnan(ld.pool).any() and not np.isnan(lc.pool).any()
    oc, od = oracle_attn(oracle, bc, lc), oracle_attn(oracle, bd, ld)
    assert np.all(np.isfinite(od))
    assert np.array_equal(oc, od)


# --- input conversions the oracle does itself ------------------------------------------
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_sixteen_bit_inputs_are_read_exactly(oracle, dtype):
    # n = 1 returns v_0 exactly: compares the C bit decoding with numpy's / the shift rule,
    # over normal, subnormal and signed values
    cfg = _cfg(batch=1, len_lo=1, len_hi=1, dtype=dtype, d_model=64, n_heads=2, head_dim=32, poison=False)
    b = wl.make_batch(cfg, np.array([1], dtype=np.int32), np.array([KV], dtype=np.uint8))
    l = wl.make_layer(b)
    vals = np.array([0.0, -0.0, 1.0, -2.5, 6.1e-5, 5.96e-8, 3.0e-6, 65504.0, -1e-3, 0.333] * 7, dtype=np.float32)[:64]
    row = wl.kv_row_view(b, l.pool, 0, 0, 1)
    row[...] = wl.round_to_dtype(vals, dtype).reshape(row.shape)
    out = oracle_attn(oracle, b, l).reshape(-1)
    assert np.array_equal(out, wl.to_f64(row, dtype).reshape(-1))


def test_bad_arguments_are_rejected(oracle):
    cfg = _cfg(batch=2, len_hi=9)
    b = wl.make_batch(cfg)
    l = wl.make_layer(b)
    bad = b.ctx_lens.copy(); bad[0] = 0
    with pytest.raises(ValueError):
        oracle.attn(oracle_shape(oracle, b), l.q, l.pool, l.pool, l.pool, l.W_K, l.b_K, l.W_V, l.b_V,
                    b.block_tables, bad, b.cache_kind)
    with pytest.raises(ValueError):
        oracle_attn(oracle, b, l, kinds=np.array([2, 0], dtype=np.uint8))


# --- partial statistics against numpy (the key bias shifts every score of a request by
# the same amount, so only the partial maximum m can show it) -----------------------------
def test_partial_statistics_match_numpy(oracle):
    cfg = _cfg(batch=2, len_lo=9, len_hi=30)
    b = wl.make_batch(cfg, cache_kind=np.array([HID, KV], dtype=np.uint8))
    l = wl.make_layer(b)
    sh = oracle_shape(oracle, b)
    qs = wl.to_f64(l.q, cfg.dtype)
    for r in range(2):
        K, V = logical_kv(b, l, r)
        n = int(b.ctx_lens[r])
        t0, t1 = 3, n - 2
        for h in range(cfg.n_heads):
            m, lsum, acc = oracle.partial(sh, l.q, l.pool, l.pool, l.pool, l.W_K, l.b_K, l.W_V, l.b_V,
                                          b.block_tables, b.cache_kind[r], r, h, t0, t1)
            s = cfg.softmax_scale * (K[t0:t1, h] @ qs[r, h])
            assert abs(m - s.max()) < 1e-12
            e = np.exp(s - s.max())
            assert abs(lsum - e.sum()) < 1e-12
            assert np.max(np.abs(acc - e @ V[t0:t1, h])) < 1e-12
