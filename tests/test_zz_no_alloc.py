"""apt_hybrid_decode_attn_static (the entry point for callers that cannot allocate: its partial
results live in a static device array of the library) against apt_hybrid_decode_attn with a caller
workspace: two calls in a row through the C ABI, the second on a smaller batch, each compared with
the existing entry point bit for bit and with the CPU oracle to the parity tolerance (max-abs 2e-3,
max-rel 1e-2).  Also: the size limit is enforced and the absorbed-weight path is refused."""
import numpy as np
import pytest
import torch

from paper_2504_07494_amd import binding as ab
from paper_2504_07494_amd import workloads as wl
from tests.helpers import oracle_attn

pytestmark = pytest.mark.gpu


def _both(batch, layer):
    from paper_2504_07494_amd.harness import DecodeRunner
    rn = DecodeRunner(batch)
    dl = rn.upload(layer)
    rn.run(dl)
    want = rn.out.clone()
    torch.cuda.synchronize()
    out = torch.full_like(rn.out, float("nan"))
    ab.apt_hybrid_decode_attn_static(rn.shape, rn.plan_host, rn.plan_dev, dl.q, dl.k_pool, dl.v_pool, dl.pool,
                                     dl.W_K, dl.W_V, dl.W_packed, dl.b_K, dl.b_V, rn.block_tables, out, rn.stream())
    torch.cuda.synchronize()
    return rn, want, out


def _check(oracle, batch, layer, want, out, label):
    assert torch.equal(want, out), f"{label}: differs from the caller-workspace entry point"
    c = batch.cfg
    ref = oracle_attn(oracle, batch, layer).reshape(batch.B, c.n_heads, c.head_dim)
    got = out.float().cpu().numpy().astype(np.float64)
    err = np.abs(got - ref)
    big = np.abs(ref) >= 1e-2
    a, r = float(err.max()), float((err[big] / np.abs(ref[big])).max())
    print(f"[parity] {label}: max_abs={a:.3e} max_rel={r:.3e}", flush=True)
    assert np.all(np.isfinite(got)) and a <= 2e-3 and r <= 1e-2


def test_static_workspace_entry_point_two_calls_second_smaller(oracle):
    print("[case] static workspace entry point", flush=True)
    ab.apt_init()
    big = wl.small_config(name="noalloc_a", dtype="f16", d_model=1024, n_heads=8, head_dim=128, block_size=16,
                          batch=12, len_lo=1, len_hi=1400, hidden_ratio=0.5)
    small = wl.small_config(name="noalloc_b", dtype="f16", d_model=1024, n_heads=8, head_dim=128, block_size=16,
                            batch=3, len_lo=1, len_hi=300, hidden_ratio=0.67)
    for cfg in (big, small):                      # the second call reuses the array the first one left dirty
        batch = wl.make_batch(cfg)
        layer = wl.make_layer(batch)
        rn, want, out = _both(batch, layer)
        assert 0 < int(rn.info.workspace_bytes) <= ab.APT_STATIC_WORKSPACE_BYTES
        _check(oracle, batch, layer, want, out, cfg.name)
    # fp32 inputs (plain-ALU hidden kernel) share the same array
    batch = wl.make_batch(wl.CONFIGS["tiny"])
    layer = wl.make_layer(batch)
    rn, want, out = _both(batch, layer)
    _check(oracle, batch, layer, want, out, "tiny")


def test_static_workspace_entry_point_rejects_what_does_not_fit(oracle):
    from paper_2504_07494_amd.harness import DecodeRunner
    # a plan whose partials exceed the static array: 512 requests x 8 ranges x 40 heads x 520 B = 85 MB
    cfg = wl.small_config(name="noalloc_big", dtype="f16", d_model=5120, n_heads=40, head_dim=128, block_size=16,
                          batch=512, len_lo=2000, len_hi=2048, hidden_ratio=1.0)
    batch = wl.make_batch(cfg)
    shape = ab.make_shape(cfg.d_model, cfg.n_heads, cfg.head_dim, cfg.block_size, cfg.dtype, batch.max_blocks,
                          cfg.softmax_scale)
    plan = np.zeros(ab.apt_plan_max_bytes(shape, batch.B, 2048) // 4, dtype=np.int32)
    info = ab.apt_plan(shape, batch.ctx_lens, batch.cache_kind, plan)
    assert int(info.workspace_bytes) > ab.APT_STATIC_WORKSPACE_BYTES
    P = 256         # any aligned non-null address: the call must fail before anything is launched
    with pytest.raises(ab.AptError) as e:
        ab.apt_hybrid_decode_attn_static(shape, plan, P, P, P, P, P, None, None, P, P, P, P, P, 0)
    assert e.value.status == ab.APT_EWORKSPACE
    # the absorbed-weight path needs a far larger workspace: refused
    small = wl.make_batch(wl.small_config(name="noalloc_c", dtype="f16", d_model=512, n_heads=4, head_dim=128,
                                          block_size=16, batch=2, len_lo=10, len_hi=40, hidden_ratio=0.5))
    rn = DecodeRunner(small, hidden_impl=ab.APT_HIDDEN_ABSORBED)
    with pytest.raises(ab.AptError) as e:
        ab.apt_hybrid_decode_attn_static(rn.shape, rn.plan_host, rn.plan_dev, P, P, P, P, P, P, None, P, P, P, P, 0)
    assert e.value.status == ab.APT_ESHAPE
