"""Device-side plumbing around the C-ABI calls: holds the torch buffers of one batch
(plan, cache maps, workspace, output) and of one layer (pool, weights, q) and issues
the library calls.  Memory and streams only; no arithmetic happens here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as ab
from . import workloads as wl

_TORCH_OUT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def _to_dev(raw: np.ndarray, device) -> torch.Tensor:
    """Upload a raw storage array byte for byte (16-bit types travel as int16)."""
    a = np.ascontiguousarray(raw)
    if a.dtype in (np.uint16, np.float16):
        a = a.view(np.int16)
    return torch.from_numpy(a).to(device)


class DeviceLayer:
    def __init__(self, runner: "DecodeRunner", layer: wl.Layer, separate_pools: bool = False,
                 keep_raw_weights: bool = True):
        dev = runner.device
        self.pool = _to_dev(layer.pool, dev)
        if separate_pools:
            self.k_pool, self.v_pool = self.pool.clone(), self.pool.clone()
        else:
            self.k_pool = self.v_pool = self.pool      # one unified pool
        self.W_K = _to_dev(layer.W_K, dev)
        self.W_V = _to_dev(layer.W_V, dev)
        self.b_K = _to_dev(layer.b_K, dev)
        self.b_V = _to_dev(layer.b_V, dev)
        self.q = _to_dev(layer.q, dev)
        self.W_packed = None
        if runner.info.hidden_impl == ab.APT_HIDDEN_MFMA:
            nbytes = ab.apt_packed_weight_bytes(runner.shape)
            self.W_packed = torch.empty(nbytes, dtype=torch.uint8, device=dev)
            ab.apt_pack_weights(runner.shape, self.W_K, self.W_V, self.W_packed,
                                torch.cuda.current_stream(dev).cuda_stream)
            if not keep_raw_weights:          # the MFMA kernel reads only the packed copy
                torch.cuda.current_stream(dev).synchronize()
                self.W_K = self.W_V = None


class DecodeRunner:
    """One batch: plan + cache maps + workspace + output buffer on the device."""

    def __init__(self, batch: wl.Batch, out_dtype: str = "f32", hidden_impl: int = ab.APT_HIDDEN_AUTO,
                 hidden_chunk: int = 0, kv_chunk: int = 0, device: str = "cuda:0", scale=None):
        if not torch.cuda.is_available():
            raise RuntimeError("a GPU is required: there is no CPU path")
        cfg = batch.cfg
        self.batch, self.cfg = batch, cfg
        self.device = torch.device(device)
        self.out_dtype = out_dtype
        self.shape = ab.make_shape(cfg.d_model, cfg.n_heads, cfg.head_dim, cfg.block_size, cfg.dtype,
                                   batch.max_blocks, cfg.softmax_scale if scale is None else scale,
                                   out_dtype=out_dtype, hidden_chunk=hidden_chunk, kv_chunk=kv_chunk,
                                   hidden_impl=hidden_impl)
        max_ctx = batch.max_blocks * cfg.block_size
        # sized once for every batch of at most B requests of this shape, whatever their lengths and kinds
        ws_bytes, plan_bytes = ab.apt_workspace_bytes(self.shape, batch.B, max_ctx)
        # The plan blob is written on the host and copied asynchronously: a host buffer is rewritten only after the
        # copy that last read it has completed (one event per buffer), so steps can be planned back to back
        # without a device synchronisation and without tearing a pending copy.
        self._plan_bufs = [torch.empty(plan_bytes // 4, dtype=torch.int32, pin_memory=True) for _ in range(2)]
        self._plan_events = [None] * len(self._plan_bufs)
        self._plan_i = 0
        self.plan_host = self._plan_bufs[0]
        self.plan_dev = torch.empty(plan_bytes // 4, dtype=torch.int32, device=self.device)
        self.block_tables = torch.from_numpy(batch.block_tables).to(self.device)
        self.out = torch.empty((batch.B, cfg.n_heads, cfg.head_dim), dtype=_TORCH_OUT[out_dtype], device=self.device)
        self.workspace = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=self.device)
        self.info = None
        ab.apt_init()
        self.plan()

    def stream(self) -> int:
        return torch.cuda.current_stream(self.device).cuda_stream

    def plan(self, ctx_lens=None, cache_kind=None):
        """a1: partition on the host, copy the blob to the device.  ctx_lens / cache_kind: this step's lengths and
        kinds (default: the batch's own); lengths must stay within what the cache maps cover."""
        ctx_lens = self.batch.ctx_lens if ctx_lens is None else np.ascontiguousarray(ctx_lens, dtype=np.int32)
        cache_kind = self.batch.cache_kind if cache_kind is None else np.ascontiguousarray(cache_kind, dtype=np.uint8)
        i = self._plan_i = (self._plan_i + 1) % len(self._plan_bufs)
        if self._plan_events[i] is not None:
            self._plan_events[i].synchronize()        # the copy out of this host buffer is done
        self.plan_host = self._plan_bufs[i]
        self.info = ab.apt_plan(self.shape, ctx_lens, cache_kind, self.plan_host)
        ab.apt_plan_upload(self.plan_host, self.plan_dev, self.stream())
        ev = torch.cuda.Event()
        ev.record(torch.cuda.current_stream(self.device))
        self._plan_events[i] = ev
        assert int(self.info.workspace_bytes) <= self.workspace.numel()
        return self.info

    def upload(self, layer: wl.Layer, separate_pools: bool = False, keep_raw_weights: bool = True) -> DeviceLayer:
        return DeviceLayer(self, layer, separate_pools, keep_raw_weights)

    def run(self, dl: DeviceLayer, ev_begin=None, ev_end=None, out=None) -> torch.Tensor:
        """a2-a4: the attention call for one layer (asynchronous on the current stream).
        ev_begin / ev_end: optional raw hipEvent_t handles recorded around the item kernel.
        out: optional output tensor of this layer (default: the runner's own buffer)."""
        out = self.out if out is None else out
        if ev_begin is None and ev_end is None:
            ab.apt_hybrid_decode_attn(self.shape, self.plan_host, self.plan_dev, dl.q, dl.k_pool, dl.v_pool, dl.pool,
                                      dl.W_K, dl.W_V, dl.W_packed, dl.b_K, dl.b_V, self.block_tables, out,
                                      self.workspace, self.workspace.numel(), self.stream())
        else:
            ab.apt_hybrid_decode_attn_timed(self.shape, self.plan_host, self.plan_dev, dl.q, dl.k_pool, dl.v_pool,
                                            dl.pool, dl.W_K, dl.W_V, dl.W_packed, dl.b_K, dl.b_V, self.block_tables,
                                            out, self.workspace, self.workspace.numel(), self.stream(),
                                            ev_begin, ev_end)
        return out

    def run_step(self, layers, outs=None):
        """One decode step over several layers: the plan is made once (lengths and cache kinds are per
        request, the same in every layer), then one attention call per layer."""
        self.plan()
        for i, dl in enumerate(layers):
            self.run(dl, out=None if outs is None else outs[i])

    def out_f64(self) -> np.ndarray:
        torch.cuda.synchronize(self.device)
        return self.out.float().cpu().numpy().astype(np.float64)
