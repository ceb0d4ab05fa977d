"""GPU parity at the full sizes of the named configurations, in the launch configuration
bench.py times: sampled (request, head) outputs against the CPU oracle (each is an
independent textbook attention the oracle computes on its own), plus properties that hold
for every element (finite, bit-reproducible, unchanged when the batch is planned again)."""
import numpy as np
import pytest

from paper_2504_07494_amd import workloads as wl
from tests.helpers import oracle_attn

pytestmark = pytest.mark.gpu


def _sample_pairs(batch, n_random, seed):
    """Shortest and longest request, lengths = 0, 1, 15 mod 16 when present, both kinds,
    plus random pairs."""
    cfg = batch.cfg
    g = np.random.default_rng(seed)
    lens, kinds = batch.ctx_lens, batch.cache_kind
    picks = []
    for kind in (wl.KIND_KV, wl.KIND_HIDDEN):
        idx = np.nonzero(kinds == kind)[0]
        if len(idx) == 0:
            continue
        picks += [idx[np.argmin(lens[idx])], idx[np.argmax(lens[idx])]]
        for rem in (0, 1, 15):
            m = idx[lens[idx] % 16 == rem]
            if len(m):
                picks.append(m[0])
    pairs = [(int(r), int(g.integers(cfg.n_heads))) for r in picks]
    flat = g.choice(batch.B * cfg.n_heads, size=n_random, replace=False)
    pairs += [(int(f // cfg.n_heads), int(f % cfg.n_heads)) for f in flat]
    return sorted(set(pairs))


def _run_and_check(oracle, cfg, n_random, max_abs=2e-3, max_rel=1e-2):
    from paper_2504_07494_amd.harness import DecodeRunner
    print(f"[case] full size {cfg.name} ratio={cfg.hidden_ratio}", flush=True)
    batch = wl.make_batch(cfg)
    layer = wl.make_layer(batch, workers=16)
    rn = DecodeRunner(batch)
    dl = rn.upload(layer)
    rn.run(dl)
    got = rn.out_f64()
    assert np.all(np.isfinite(got))
    pairs = _sample_pairs(batch, n_random, cfg.seed)
    want = oracle_attn(oracle, batch, layer, pairs=pairs)
    sel = got[[p[0] for p in pairs], [p[1] for p in pairs]]
    err = np.abs(sel - want)
    big = np.abs(want) >= 1e-2
    a, r = float(err.max()), float((err[big] / np.abs(want[big])).max())
    print(f"[parity] {cfg.name}: {len(pairs)} pairs, max_abs={a:.3e} max_rel={r:.3e}", flush=True)
    assert a <= max_abs and r <= max_rel
    rn.workspace.fill_(0xFF)
    rn.plan()
    rn.run(dl)
    assert np.array_equal(rn.out_f64(), got)
    return batch, got


def test_opt13b_layer(oracle):
    _run_and_check(oracle, wl.CONFIGS["opt13b"], n_random=24)


def test_opt30b_layer_permuted_pages(oracle):
    _run_and_check(oracle, wl.CONFIGS["opt30b"], n_random=16)


@pytest.mark.parametrize("ratio", [0.0, 0.5, 1.0])
def test_opt66b_layer_ratio_sweep(oracle, ratio):
    _run_and_check(oracle, wl.with_ratio(wl.CONFIGS["opt66b"], ratio), n_random=10)
