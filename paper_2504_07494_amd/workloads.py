"""Seeded synthetic inputs for the hybrid-cache decode attention step.

This module only draws random numbers and lays them out in memory: request
lengths, per-request cache kinds, cache maps (block tables) into one unified
block pool, the pool's contents, projection weights, biases and queries.  It
holds none of the method's arithmetic (no projection, no softmax) and is the one
piece shared by the CPU oracle's tests and the GPU path's tests.

Shapes follow the paper's OPT-family setup (Section 6.2, Table 2: OPT-13B/30B/66B,
FP16, 2048-token limit), its block-wise scattered cache storage (Section 2.2) and
the unified pool in which a block holds either K, V or input-hidden vectors of a
fixed number of token positions (Section 4.3).  The paper's request traces are not
used: lengths are drawn from the stated distributions instead.

Memory layout written here (and documented in include/apt_hybrid.h):

* pool:            [n_pool_blocks][block_size * d_model] elements
* hidden block:    [slot][d_model]                (token-major rows)
* K block/V block: [head][slot][head_dim]         (head-major)
* block_tables:    int32 [B][2][max_blocks]; row 0 = K blocks (KV kind) or hidden
                   blocks (hidden kind); row 1 = V blocks (KV kind only); unused = -1
* W_K, W_V:        [d_in][d_out] row-major, k = x @ W + b
* q:               [B][H][head_dim]
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np

KIND_KV = 0
KIND_HIDDEN = 1

DTYPE_CODES = {"f32": 0, "f16": 1, "bf16": 2}
ELEM_BYTES = {"f32": 4, "f16": 2, "bf16": 2}

BASE_SEED = 250407494 * 10


# ----------------------------------------------------------------------------
# dtype helpers: 16-bit types are kept as raw arrays (float16, or uint16 bit
# patterns for bf16) so they can be handed to C by pointer.
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    nan = np.isnan(a)
    r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)
    if nan.any():
        r[nan] = np.uint16(0x7FC0)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_dtype(a32: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values once to the storage dtype (raw representation)."""
    if dtype == "f32":
        return np.ascontiguousarray(a32, dtype=np.float32)
    if dtype == "f16":
        return a32.astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(a32)
    raise ValueError(dtype)


def to_f64(raw: np.ndarray, dtype: str) -> np.ndarray:
    """Exact conversion of a raw storage array to float64."""
    if dtype == "bf16":
        return bf16_bits_to_f32(raw).astype(np.float64)
    return raw.astype(np.float64)


def raw_np_dtype(dtype: str):
    return {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}[dtype]


def nan_raw(dtype: str):
    if dtype == "bf16":
        return np.uint16(0x7FC0)
    return raw_np_dtype(dtype)(np.nan)


# ----------------------------------------------------------------------------
# counter-based streams: every tensor (and every chunk of a big tensor) has its
# own Philox key, so any slice can be regenerated alone and the result does not
# depend on the number of worker threads.
# ----------------------------------------------------------------------------
T_LENS, T_KIND, T_PAGES, T_POOL, T_WK, T_WV, T_BK, T_BV, T_Q = range(9)


def _rng(seed: int, tensor: int, layer: int = 0, chunk: int = 0) -> np.random.Generator:
    key = (np.uint64(seed & 0xFFFFFFFFFFFFFFFF), np.uint64((tensor << 48) | (layer << 32) | chunk))
    return np.random.Generator(np.random.Philox(key=np.array(key, dtype=np.uint64)))


def _normal_raw(seed, tensor, layer, shape, std, dtype, chunk_rows=None, workers=8) -> np.ndarray:
    """N(0, std^2) of `shape`, rounded to dtype; generated in row chunks on threads."""
    rows = shape[0]
    rest = int(np.prod(shape[1:])) if len(shape) > 1 else 1
    out = np.empty(shape, dtype=raw_np_dtype(dtype))
    flat = out.reshape(rows, rest)
    if chunk_rows is None:
        chunk_rows = max(1, (1 << 22) // max(rest, 1))
    n_chunks = (rows + chunk_rows - 1) // chunk_rows

    def work(c):
        lo, hi = c * chunk_rows, min(rows, (c + 1) * chunk_rows)
        g = _rng(seed, tensor, layer, c)
        x = g.standard_normal((hi - lo, rest), dtype=np.float32)
        if std != 1.0:
            x *= np.float32(std)
        flat[lo:hi] = round_to_dtype(x, dtype)

    if n_chunks == 1 or workers <= 1:
        for c in range(n_chunks):
            work(c)
    else:
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(work, range(n_chunks)))
    return out


# ----------------------------------------------------------------------------
# configuration
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class Config:
    name: str
    d_model: int
    n_heads: int
    head_dim: int
    dtype: str
    batch: int
    len_dist: str            # "uniform" | "lognormal"
    len_lo: int
    len_hi: int
    hidden_ratio: float      # share of requests on the hidden cache
    kind_rule: str = "ratio"  # "ratio" (round-half-up share, seeded shuffle) | "bernoulli"
    block_size: int = 16
    permute_pages: bool = False
    lognormal_median: float = 512.0
    lognormal_sigma: float = 1.0
    n_layers: int = 1
    w_std: float = 0.02
    seed: int = BASE_SEED
    spare_block_frac: float = 0.03   # unreferenced blocks left in the pool
    poison: bool = True              # NaN in unreferenced blocks and unused tail slots

    @property
    def softmax_scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)

    @property
    def max_blocks(self) -> int:
        return (self.len_hi + self.block_size - 1) // self.block_size

    @property
    def kv_std(self) -> float:
        # K/V pages of KV-kind requests have the distribution that x @ W + b would
        # have for x ~ N(0,1), W, b ~ N(0, w_std^2): variance d*w_std^2 + w_std^2.
        return math.sqrt(self.d_model * self.w_std ** 2 + self.w_std ** 2)


CONFIGS: Dict[str, Config] = {
    # Tiny single layer (parity only).
    "tiny": Config("tiny", 256, 4, 64, "f32", 4, "uniform", 16, 128, 0.5, seed=BASE_SEED + 1),
    # OPT-13B-shaped layer: the configuration the headline metric is quoted on.
    "opt13b": Config("opt13b", 5120, 40, 128, "f16", 64, "uniform", 128, 2048, 0.5, seed=BASE_SEED + 2),
    # OPT-30B-shaped layer, lognormal lengths, permuted physical pages.
    "opt30b": Config("opt30b", 7168, 56, 128, "f16", 128, "lognormal", 32, 2048, 0.7,
                     permute_pages=True, seed=BASE_SEED + 3),
    # OPT-66B-shaped layer; hidden ratio swept 0/25/50/75/100 % via with_ratio().
    "opt66b": Config("opt66b", 9216, 72, 128, "f16", 256, "uniform", 64, 2048, 0.5, seed=BASE_SEED + 4),
    # 40-layer OPT-13B-shaped decode step, bf16, Bernoulli(0.5) kinds shared by layers.
    "opt13b_step": Config("opt13b_step", 5120, 40, 128, "bf16", 384, "uniform", 256, 1024, 0.5,
                          kind_rule="bernoulli", n_layers=40, seed=BASE_SEED + 5),
}


def with_ratio(cfg: Config, ratio: float) -> Config:
    return replace(cfg, hidden_ratio=float(ratio))


# ----------------------------------------------------------------------------
# batch metadata: lengths, kinds, cache maps
# ----------------------------------------------------------------------------
def draw_ctx_lens(cfg: Config) -> np.ndarray:
    g = _rng(cfg.seed, T_LENS)
    if cfg.len_dist == "uniform":
        n = g.integers(cfg.len_lo, cfg.len_hi + 1, size=cfg.batch)
    elif cfg.len_dist == "lognormal":
        z = g.standard_normal(cfg.batch)
        n = np.rint(np.exp(math.log(cfg.lognormal_median) + cfg.lognormal_sigma * z))
        n = np.clip(n, cfg.len_lo, cfg.len_hi)
    else:
        raise ValueError(cfg.len_dist)
    return n.astype(np.int32)


def draw_cache_kind(cfg: Config) -> np.ndarray:
    g = _rng(cfg.seed, T_KIND)
    kind = np.zeros(cfg.batch, dtype=np.uint8)
    if cfg.kind_rule == "ratio":
        # The first k requests of one seeded shuffle are hidden-kind, so the sets of
        # a ratio sweep are nested.
        order = g.permutation(cfg.batch)
        k = int(math.floor(cfg.hidden_ratio * cfg.batch + 0.5))
        kind[order[:k]] = KIND_HIDDEN
    elif cfg.kind_rule == "bernoulli":
        kind[g.random(cfg.batch) < cfg.hidden_ratio] = KIND_HIDDEN
    else:
        raise ValueError(cfg.kind_rule)
    return kind


def blocks_needed(ctx_lens: np.ndarray, cache_kind: np.ndarray, bs: int) -> int:
    nb = (ctx_lens.astype(np.int64) + bs - 1) // bs
    return int(np.sum(np.where(cache_kind == KIND_KV, 2 * nb, nb)))


def build_block_tables(cfg: Config, ctx_lens: np.ndarray, cache_kind: np.ndarray,
                       max_blocks: Optional[int] = None):
    """Cache maps into one unified pool (Section 4.3).

    Returns (block_tables int32[B][2][max_blocks], n_pool_blocks, block_type int8[n_pool])
    with block_type 0 = unreferenced, 1 = K, 2 = V, 3 = hidden.
    """
    bs = cfg.block_size
    B = len(ctx_lens)
    if max_blocks is None:
        max_blocks = cfg.max_blocks
    need = blocks_needed(ctx_lens, cache_kind, bs)
    n_pool = need + max(1, int(math.ceil(need * cfg.spare_block_frac)))
    if cfg.permute_pages:
        ids = _rng(cfg.seed, T_PAGES).permutation(n_pool).astype(np.int32)
    else:
        ids = np.arange(n_pool, dtype=np.int32)
    bt = np.full((B, 2, max_blocks), -1, dtype=np.int32)
    btype = np.zeros(n_pool, dtype=np.int8)
    cur = 0
    for r in range(B):
        nb = (int(ctx_lens[r]) + bs - 1) // bs
        if nb > max_blocks:
            raise ValueError("context longer than max_blocks * block_size")
        bt[r, 0, :nb] = ids[cur:cur + nb]
        if cache_kind[r] == KIND_KV:
            btype[ids[cur:cur + nb]] = 1
            cur += nb
            bt[r, 1, :nb] = ids[cur:cur + nb]
            btype[ids[cur:cur + nb]] = 2
            cur += nb
        else:
            btype[ids[cur:cur + nb]] = 3
            cur += nb
    assert cur == need
    return bt, n_pool, btype


@dataclass
class Batch:
    """Metadata shared by all layers of one decode step."""
    cfg: Config
    ctx_lens: np.ndarray       # int32 [B]
    cache_kind: np.ndarray     # uint8 [B]
    block_tables: np.ndarray   # int32 [B][2][max_blocks]
    n_pool_blocks: int
    block_type: np.ndarray     # int8 [n_pool_blocks]
    max_blocks: int

    @property
    def B(self) -> int:
        return len(self.ctx_lens)

    @property
    def total_tokens(self) -> int:
        return int(self.ctx_lens.astype(np.int64).sum())

    @property
    def hidden_tokens(self) -> int:
        return int(self.ctx_lens[self.cache_kind == KIND_HIDDEN].astype(np.int64).sum())

    @property
    def kv_tokens(self) -> int:
        return self.total_tokens - self.hidden_tokens


def make_batch(cfg: Config, ctx_lens: Optional[np.ndarray] = None,
               cache_kind: Optional[np.ndarray] = None) -> Batch:
    if ctx_lens is None:
        ctx_lens = draw_ctx_lens(cfg)
    ctx_lens = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    if cache_kind is None:
        cache_kind = draw_cache_kind(replace(cfg, batch=len(ctx_lens)))
    cache_kind = np.ascontiguousarray(cache_kind, dtype=np.uint8)
    max_blocks = max(cfg.max_blocks, int((ctx_lens.max() + cfg.block_size - 1) // cfg.block_size))
    bt, n_pool, btype = build_block_tables(cfg, ctx_lens, cache_kind, max_blocks)
    return Batch(cfg, ctx_lens, cache_kind, bt, n_pool, btype, max_blocks)


# ----------------------------------------------------------------------------
# per-layer tensors
# ----------------------------------------------------------------------------
@dataclass
class Layer:
    pool: np.ndarray   # raw [n_pool_blocks][bs*d]
    W_K: np.ndarray    # raw [d][d]
    W_V: np.ndarray
    b_K: np.ndarray    # raw [d]
    b_V: np.ndarray
    q: np.ndarray      # raw [B][H][hd]
    extra: dict = field(default_factory=dict)


def fill_pool(batch: Batch, layer: int = 0, workers: int = 8) -> np.ndarray:
    """Pool contents: hidden blocks ~ N(0,1), K/V blocks ~ N(0, kv_std^2); with
    cfg.poison, unreferenced blocks and the unused slots of last blocks are NaN."""
    cfg = batch.cfg
    bs, d, H, hd = cfg.block_size, cfg.d_model, cfg.n_heads, cfg.head_dim
    n_pool = batch.n_pool_blocks
    blk = bs * d
    pool = np.empty((n_pool, blk), dtype=raw_np_dtype(cfg.dtype))
    scale = np.where(batch.block_type == 3, 1.0, cfg.kv_std).astype(np.float32)
    chunk = max(1, (1 << 23) // blk)
    n_chunks = (n_pool + chunk - 1) // chunk

    def work(c):
        lo, hi = c * chunk, min(n_pool, (c + 1) * chunk)
        g = _rng(cfg.seed, T_POOL, layer, c)
        x = g.standard_normal((hi - lo, blk), dtype=np.float32)
        x *= scale[lo:hi, None]
        pool[lo:hi] = round_to_dtype(x, cfg.dtype)

    if n_chunks == 1 or workers <= 1:
        for c in range(n_chunks):
            work(c)
    else:
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(work, range(n_chunks)))

    if cfg.poison:
        nanv = nan_raw(cfg.dtype)
        pool[batch.block_type == 0] = nanv
        for r in range(batch.B):
            n = int(batch.ctx_lens[r])
            used = n % bs
            if used == 0:
                continue
            last = (n - 1) // bs
            if batch.cache_kind[r] == KIND_HIDDEN:
                b = int(batch.block_tables[r, 0, last])
                pool[b].reshape(bs, d)[used:] = nanv
            else:
                for row in (0, 1):
                    b = int(batch.block_tables[r, row, last])
                    pool[b].reshape(H, bs, hd)[:, used:, :] = nanv
    return pool


def make_layer(batch: Batch, layer: int = 0, workers: int = 8) -> Layer:
    cfg = batch.cfg
    d, H, hd = cfg.d_model, cfg.n_heads, cfg.head_dim
    s, dt = cfg.seed, cfg.dtype
    return Layer(
        pool=fill_pool(batch, layer, workers),
        W_K=_normal_raw(s, T_WK, layer, (d, d), cfg.w_std, dt, workers=workers),
        W_V=_normal_raw(s, T_WV, layer, (d, d), cfg.w_std, dt, workers=workers),
        b_K=_normal_raw(s, T_BK, layer, (d,), cfg.w_std, dt, workers=1),
        b_V=_normal_raw(s, T_BV, layer, (d,), cfg.w_std, dt, workers=1),
        q=_normal_raw(s, T_Q, layer, (batch.B, H, hd), 1.0, dt, workers=1),
    )


def small_config(name: str = "small", **kw) -> Config:
    """A config for unit tests; keyword overrides on top of a tiny fp32 base."""
    base = dict(name=name, d_model=64, n_heads=2, head_dim=32, dtype="f32", batch=3,
                len_dist="uniform", len_lo=1, len_hi=40, hidden_ratio=0.5, block_size=4,
                seed=BASE_SEED + 99)
    base.update(kw)
    return Config(**base)


# ----------------------------------------------------------------------------
# layout accessors (pure indexing, used by tests to read or write logical rows)
# ----------------------------------------------------------------------------
def hidden_row_view(batch: Batch, pool: np.ndarray, r: int, j: int) -> np.ndarray:
    """View of x_j (d elements) of hidden-kind request r."""
    cfg = batch.cfg
    b = int(batch.block_tables[r, 0, j // cfg.block_size])
    return pool[b].reshape(cfg.block_size, cfg.d_model)[j % cfg.block_size]


def kv_row_view(batch: Batch, pool: np.ndarray, r: int, j: int, which: int) -> np.ndarray:
    """View [H][hd] of k_j (which=0) or v_j (which=1) of KV-kind request r."""
    cfg = batch.cfg
    b = int(batch.block_tables[r, which, j // cfg.block_size])
    return pool[b].reshape(cfg.n_heads, cfg.block_size, cfg.head_dim)[:, j % cfg.block_size, :]
