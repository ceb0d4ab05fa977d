"""The attention call inside a HIP graph: it launches kernels on the caller's stream only (no
allocation, no synchronisation, no memset nodes), so it can be captured once and replayed.  Every
replay is compared with the eager call on the same inputs, with eager work and synchronisations
between the replays."""
import numpy as np
import pytest
import torch

from paper_2504_07494_amd import binding as ab
from paper_2504_07494_amd import workloads as wl

pytestmark = pytest.mark.gpu

KV, HID = wl.KIND_KV, wl.KIND_HIDDEN


@pytest.mark.parametrize("impl", [ab.APT_HIDDEN_AUTO, ab.APT_HIDDEN_ABSORBED])
def test_captured_attention_call_replays_like_the_eager_call(oracle, impl):
    from paper_2504_07494_amd.harness import DecodeRunner, _to_dev
    print(f"[case] graph capture hidden_impl={impl}", flush=True)
    cfg = wl.small_config(name="graph", dtype="f16", d_model=512, n_heads=4, head_dim=128, block_size=16,
                          batch=6, len_lo=1, len_hi=900, hidden_ratio=0.5)
    batch = wl.make_batch(cfg, np.array([900, 257, 1, 512, 513, 33], dtype=np.int32),
                          np.array([HID, HID, HID, KV, KV, KV], dtype=np.uint8))
    layer = wl.make_layer(batch)
    rn = DecodeRunner(batch, hidden_impl=impl)
    dl = rn.upload(layer)
    rn.run(dl)                                   # eager warm-up (one-off function attributes are set here)
    torch.cuda.synchronize()
    g = np.random.default_rng(3)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    out_graph = torch.empty_like(rn.out)
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            rn.run(dl, out=out_graph)            # uses the capturing stream (torch's current stream)
    torch.cuda.synchronize()
    for rep in range(4):
        q = wl.round_to_dtype(g.standard_normal((batch.B, cfg.n_heads, cfg.head_dim), dtype=np.float32), cfg.dtype)
        dl.q.copy_(_to_dev(q, rn.device))        # new queries in the captured buffer
        eager = rn.run(dl).clone()
        torch.cuda.synchronize()
        out_graph.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_graph, eager), rep
        assert bool(torch.isfinite(out_graph).all())
    # and the last replay against the oracle
    layer.q[...] = q
    from tests.helpers import oracle_attn
    want = oracle_attn(oracle, batch, layer).reshape(batch.B, cfg.n_heads, cfg.head_dim)
    assert np.max(np.abs(out_graph.float().cpu().numpy().astype(np.float64) - want)) < 2e-4
