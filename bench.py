#!/usr/bin/env python3
"""Benchmark of the hybrid-cache decode attention step on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W [--config opt66b] [--hidden-ratio R]

A step is one pass of the whole hot path for one layer over one synthetic batch whose
inputs are already resident in HBM: the ragged work partition (host planner + copy of the
plan to the device), the item kernel (paged-KV attention and hidden-cache recompute +
attention in one launch) and the merge kernel.  The metric is cached tokens per second
per decode layer = sum of the batch's context lengths / time per step.

Default run (no flags): the OPT-66B-shaped layer (batch 256), the largest single-layer
configuration.  The headline `value`, `roofline` and `cpu_baseline` are its 50 % hidden-cache
point; `sweep` holds the hidden-cache ratios 0/25/50/75/100 % of the same batch (0 % is the
HBM-bound point, 100 % the MFMA-bound one), each timed with the same W warm-up and K timed
steps; `rho_fit` is the least-squares line of the item-kernel time over the hidden tokens
(Section 4.2, Eq. 5-6: t = rho * m); `other_configs` adds the OPT-13B- and OPT-30B-shaped
layers and the 40-layer OPT-13B-shaped step (--no-extras skips them).

Prints ONE JSON line.  `roofline` describes the item kernel, timed with HIP events
recorded around it on its launch stream inside the timed region.  `cpu_baseline` is the
CPU oracle timed on this machine's host cores over a bounded random sample of (request,
head) pairs of the same batch (it is a baseline, not a target); the same sample is used
to check the GPU output.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_HBM_GBS = 8000.0
PEAK_MFMA_TFLOPS = {"f16": 2500.0, "bf16": 2500.0, "f32": 157.3}
# the absorbed-weight hidden path (opt-in, not the paper's method) reads every cached hidden row twice
ABSORBED_X_READS = 2.0


class HipEvents:
    """Pairs of raw HIP events (created through the HIP runtime that torch has loaded)."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.pairs = []
        for _ in range(n):
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(a)) == 0
            assert self.hip.hipEventCreate(ctypes.byref(b)) == 0
            self.pairs.append((a, b))

    def elapsed_ms(self, i):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.pairs[i][0], self.pairs[i][1])
        assert rc == 0, rc
        return ms.value

    def close(self):
        for a, b in self.pairs:
            self.hip.hipEventDestroy(a)
            self.hip.hipEventDestroy(b)


def read_traffic(workload_key):
    """HBM bytes per item-kernel launch measured with rocprofv3 --pmc (FETCH_SIZE and
    WRITE_SIZE, scaled by a copy kernel of known size), kept as text under profiles/."""
    path = os.path.join(ROOT, "profiles", "traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        t = line.split()
        if len(t) >= 2 and t[0] == workload_key:
            try:
                return float(t[1])
            except ValueError:
                return None
    return None


HIMPL = {"auto": 0, "valu": 1, "mfma": 2, "absorbed": 3}


def measure(cfg, args, steps, warmup, keep=False):
    """W warm-up steps, then K timed steps (plan + plan copy + one attention call per layer) of one workload,
    bracketed by device synchronisations.  Returns a dict of the measured numbers; with keep=True also the
    runner, the batch and the last layer's host copy (for the oracle sample)."""
    import numpy as np
    import torch
    from paper_2504_07494_amd import workloads as wl
    from paper_2504_07494_amd.harness import DecodeRunner

    t_gen = time.time()
    batch = wl.make_batch(cfg)
    nl = cfg.n_layers
    himpl = HIMPL[args.hidden_impl]
    rn = DecodeRunner(batch, kv_chunk=args.kv_chunk, hidden_chunk=args.hidden_chunk, hidden_impl=himpl)
    layer, dls = None, []
    for li in range(nl):                      # every layer of the step is resident in HBM
        layer = wl.make_layer(batch, layer=li, workers=min(16, os.cpu_count() or 8))
        dls.append(rn.upload(layer, keep_raw_weights=(nl == 1 or himpl == 3)))
    t_gen = time.time() - t_gen
    torch.cuda.synchronize()

    for _ in range(warmup):
        rn.run_step(dls)
    torch.cuda.synchronize()

    ev = HipEvents(steps * nl)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        rn.plan()
        for li in range(nl):
            rn.run(dls[li], ev.pairs[i * nl + li][0], ev.pairs[i * nl + li][1])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    kern_ms = [ev.elapsed_ms(i) for i in range(steps * nl)]
    ev.close()
    kern_avg_ms = float(np.mean(kern_ms))

    total_tokens, hidden_tokens, kv_tokens = batch.total_tokens, batch.hidden_tokens, batch.kv_tokens
    d, e = cfg.d_model, wl.ELEM_BYTES[cfg.dtype]
    # algorithmic work of the item kernel per launch
    flops = 4.0 * d * d * hidden_tokens                 # K and V projections of hidden-kind tokens
    kv_bytes = 2.0 * d * e * kv_tokens                  # K row + V row of KV-kind tokens
    hid_bytes = 1.0 * d * e * hidden_tokens
    absorbed = int(rn.info.hidden_impl) == 3 and hidden_tokens > 0
    if absorbed:
        # absorbed form: no projection; per hidden token and head one d_model-long dot product and one
        # d_model-long weighted row update (4 d H flops); priced against HBM, on its own bytes
        flops = 4.0 * d * cfg.n_heads * hidden_tokens
        hid_bytes = ABSORBED_X_READS * d * e * hidden_tokens
    t_mfma = flops / (PEAK_MFMA_TFLOPS[cfg.dtype] * 1e12)
    t_hbm = (kv_bytes + hid_bytes) / (PEAK_HBM_GBS * 1e9)
    wkey = f"{cfg.name}@{cfg.hidden_ratio:g}" + ("@absorbed" if absorbed else "")
    tflops = flops / (kern_avg_ms * 1e-3) / 1e12
    gbs = (kv_bytes + hid_bytes) / (kern_avg_ms * 1e-3) / 1e9
    if not absorbed and t_mfma >= t_hbm:
        roof = {"bound": "mfma", "achieved": tflops, "peak": PEAK_MFMA_TFLOPS[cfg.dtype], "unit": "TFLOP/s",
                "frac": tflops / PEAK_MFMA_TFLOPS[cfg.dtype], "traffic": read_traffic(wkey)}
    else:
        roof = {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": gbs / PEAK_HBM_GBS, "traffic": read_traffic(wkey)}
    mfma_items = rn.info.n_hidden_items > 0 and rn.info.hidden_impl == 2
    kname = "apt_items_mfma_kernel" if mfma_items else "apt_items_kernel"
    if absorbed:
        kname = "apt_absorb_{q,score,stats,pv,out,final}_kernel + apt_items_kernel (one event pair around all of them)"
    roof.update({"kernel": kname, "kernel_ms": kern_avg_ms, "kernel_ms_min": float(np.min(kern_ms)),
                 "algorithmic_flops": flops, "algorithmic_bytes": kv_bytes + hid_bytes})
    m = {
        # cached tokens per second per decode layer: a step of nl layers serves total_tokens in each layer
        "value": total_tokens * nl / (ms_per_step * 1e-3), "ms_per_step": ms_per_step, "roofline": roof,
        "workload": f"{cfg.name}: d_model={d}, {cfg.n_heads} heads x {cfg.head_dim}, {cfg.dtype}, "
                    f"batch {batch.B}, ctx {cfg.len_dist}[{cfg.len_lo},{cfg.len_hi}], block {cfg.block_size}, "
                    f"{int(round(100 * cfg.hidden_ratio))}% hidden-cache requests"
                    + (f", {nl} layers per step (one plan, {nl} attention calls)" if nl > 1 else ""),
        "config": {"layers_per_step": nl, "total_tokens": total_tokens, "hidden_tokens": hidden_tokens,
                   "kv_tokens": kv_tokens,
                   "hidden_impl": {1: "valu", 2: "mfma", 3: "absorbed"}[int(rn.info.hidden_impl)],
                   "n_items": int(rn.info.n_items), "n_hidden_items": int(rn.info.n_hidden_items),
                   "seed": cfg.seed, "input_gen_s": round(t_gen, 2)},
        "mfma_frac": None if absorbed else tflops / PEAK_MFMA_TFLOPS[cfg.dtype],
        "hbm_frac": gbs / PEAK_HBM_GBS, "dtype": cfg.dtype,
    }
    if keep:
        m["_keep"] = (rn, batch, layer, dls)
    else:
        del rn, dls, layer
        torch.cuda.empty_cache()
    return m


def absorbed_context(batch, layer, rn, args):
    """Context only: the same step with hidden-kind requests through the absorbed-weight form (no K/V
    projection: not the paper's method, so it is never the headline and never priced in projection flops)."""
    import torch
    from paper_2504_07494_amd import workloads as wl
    from paper_2504_07494_amd.harness import DecodeRunner
    cfg = batch.cfg
    d, e = cfg.d_model, wl.ELEM_BYTES[cfg.dtype]
    total_tokens, hidden_tokens, kv_tokens = batch.total_tokens, batch.hidden_tokens, batch.kv_tokens
    rn2 = DecodeRunner(batch, kv_chunk=args.kv_chunk, hidden_impl=3)
    dl2 = rn2.upload(layer)
    for _ in range(3):
        rn2.plan()
        rn2.run(dl2)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(args.steps):
        rn2.plan()
        rn2.run(dl2)
    torch.cuda.synchronize()
    ms2 = (time.perf_counter() - t2) * 1e3 / args.steps
    dev = float((rn2.out.float() - rn.out.float()).abs().max())
    out = {
        "ms_per_step": ms2, "cached_tokens_per_s": total_tokens / (ms2 * 1e-3),
        "max_abs_difference_to_default_path": dev,
        "hbm_frac_on_own_bytes": (2.0 * d * e * kv_tokens + ABSORBED_X_READS * d * e * hidden_tokens) / (ms2 * 1e-3) / 1e9 / PEAK_HBM_GBS}
    del rn2, dl2
    return out


def resident_bytes(cfg):
    """HBM a workload keeps resident: per layer its block pool and both forms of the weights."""
    from paper_2504_07494_amd import workloads as wl
    e = wl.ELEM_BYTES[cfg.dtype]
    batch = wl.make_batch(cfg)                               # lengths, kinds and cache maps only: cheap
    pool = float(batch.n_pool_blocks) * cfg.block_size * cfg.d_model * e
    return cfg.n_layers * (pool + 4.0 * cfg.d_model ** 2 * e)


def sweep_row(ratio, m):
    r = m["roofline"]
    row = {"hidden_ratio": ratio, "total_tokens": m["config"]["total_tokens"], "hidden_tokens": m["config"]["hidden_tokens"],
           "ms_per_step": m["ms_per_step"], "kernel_ms": r["kernel_ms"], "cached_tokens_per_s": m["value"],
           "bound": r["bound"], "hbm_gbs": m["hbm_frac"] * PEAK_HBM_GBS, "hbm_frac": m["hbm_frac"]}
    if m["mfma_frac"] is not None:        # the absorbed form does no projection: never priced in projection flops
        row.update({"mfma_tflops": m["mfma_frac"] * PEAK_MFMA_TFLOPS[m["dtype"]], "mfma_frac": m["mfma_frac"]})
    return row


def brief(m):
    r = m["roofline"]
    return {"workload": m["workload"], "cached_tokens_per_s": m["value"], "ms_per_step": m["ms_per_step"],
            "kernel_ms": r["kernel_ms"], "bound": r["bound"], "roofline_frac": r["frac"], "mfma_frac": m["mfma_frac"],
            "hbm_frac": m["hbm_frac"], "total_tokens": m["config"]["total_tokens"],
            "hidden_tokens": m["config"]["hidden_tokens"], "layers_per_step": m["config"]["layers_per_step"],
            "input_gen_s": m["config"]["input_gen_s"]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="opt66b")
    ap.add_argument("--hidden-ratio", type=float, default=None)
    ap.add_argument("--kv-chunk", type=int, default=0)
    ap.add_argument("--hidden-chunk", type=int, default=0,
                    help="tokens per hidden-kind work item (0 = library default; the MFMA kernel has tiles of 256 and 320)")
    ap.add_argument("--hidden-impl", choices=["auto", "valu", "mfma", "absorbed"], default="auto",
                    help="hidden-kind kernel; 'absorbed' is the re-associated form without K/V projection (its "
                         "roofline entry is priced on its own work, never against the MFMA target)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-next-rows", action="store_true",
                    help="skip the short extra measurement of the absorbed-weight hidden path (single-layer runs "
                         "of the default hidden path add it under 'next_rows'; it never enters 'value')")
    ap.add_argument("--pairs-per-thread", type=int, default=48)
    ap.add_argument("--model-layers", type=int, default=64,
                    help="decoder layers of the model the layer shape belongs to (OPT-66B: 64); only scales the fitted "
                         "slope into the per-request rho that the scheduling example under 'next_rows' uses")
    ap.add_argument("--sweep", dest="sweep", action="store_true", default=None,
                    help="time hidden-cache ratios 0/25/50/75/100 %% of the config (adds 'sweep' and 'rho_fit'); "
                         "on by default for the default config when no --hidden-ratio is given")
    ap.add_argument("--no-sweep", dest="sweep", action="store_false")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the other configurations (opt13b, opt30b, the 40-layer opt13b_step) of the default run")
    ap.add_argument("--probe", choices=["copy", "mfma", "sched"], default=None,
                    help="run only a calibration kernel (plain copy of 1 GiB, or the register-only MFMA loop), or time "
                         "the host-side greedy scheduler at the candidate counts of the paper's scalability table")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1")

    import numpy as np
    import torch
    from paper_2504_07494_amd import workloads as wl
    from paper_2504_07494_amd.harness import DecodeRunner

    if args.probe == "sched":
        return run_sched_probe(args)
    if args.probe:
        return run_probe(args)

    default_run = args.config == "opt66b" and args.hidden_ratio is None and args.hidden_impl == "auto"
    do_sweep = args.sweep if args.sweep is not None else default_run
    do_extras = default_run and not args.no_extras
    cfg = wl.CONFIGS[args.config]
    if args.hidden_ratio is not None:
        cfg = wl.with_ratio(cfg, args.hidden_ratio)
    nl = cfg.n_layers

    sweep = []
    if do_sweep and nl == 1:
        # the ratios other than the headline's first, so that the headline's buffers can stay for the oracle sample
        for r in (0.0, 0.25, 0.5, 0.75, 1.0):
            if abs(r - cfg.hidden_ratio) > 1e-9:
                sweep.append(sweep_row(r, measure(wl.with_ratio(cfg, r), args, args.steps, args.warmup)))
    head = measure(cfg, args, args.steps, args.warmup, keep=True)
    rn, batch, layer, dls = head.pop("_keep")
    if do_sweep and nl == 1:
        sweep.append(sweep_row(cfg.hidden_ratio, head))
        sweep.sort(key=lambda p: p["hidden_ratio"])
    total_tokens, hidden_tokens, kv_tokens = batch.total_tokens, batch.hidden_tokens, batch.kv_tokens
    d, e = cfg.d_model, wl.ELEM_BYTES[cfg.dtype]
    himpl = HIMPL[args.hidden_impl]

    roof = head["roofline"]
    if roof["bound"] == "mfma":
        roof["target_frac"] = 0.50
        roof["note"] = ("MFMA fraction of the published dense peak on un-padded projection flops 4 d^2 per hidden token; "
                        + ("below" if roof["frac"] < 0.5 else "at or above") + " the 0.50 target")
    result = {
        "metric": "cached tokens/sec per decode layer; HBM GB/s and MFMA util vs MI355X peak",
        "value": head["value"], "unit": "cached tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": dict({"workload": head["workload"]}, **head["config"]),
        "roofline": roof,
    }

    if not args.no_cpu_baseline:
        from oracle import oracle as o
        nthreads = o.threads()
        g = np.random.default_rng(cfg.seed)
        n_pairs = min(batch.B * cfg.n_heads, args.pairs_per_thread * nthreads)
        flat = g.choice(batch.B * cfg.n_heads, size=n_pairs, replace=False)
        pairs = np.stack([flat // cfg.n_heads, flat % cfg.n_heads], axis=1).astype(np.int32)
        sh = o.shape_of(d, cfg.n_heads, cfg.head_dim, cfg.block_size, cfg.dtype, batch.max_blocks, cfg.softmax_scale)
        tc = time.perf_counter()
        want = o.attn(sh, layer.q, layer.pool, layer.pool, layer.pool, layer.W_K, layer.b_K, layer.W_V, layer.b_V,
                      batch.block_tables, batch.ctx_lens, batch.cache_kind, pairs=pairs)
        tc = time.perf_counter() - tc
        tok_equiv = float(batch.ctx_lens[pairs[:, 0]].astype(np.int64).sum()) / cfg.n_heads
        got = rn.out_f64()[pairs[:, 0], pairs[:, 1]]
        err = np.abs(got - want)
        big = np.abs(want) >= 1e-2
        result["cpu_baseline"] = {
            "value": tok_equiv / tc, "unit": "cached tokens/s", "cores": nthreads, "kind": "oracle",
            "sample": f"{n_pairs} random (request, head) pairs of the same batch = {tok_equiv:.0f} token-equivalents "
                      f"in {tc:.1f} s, extrapolated",
        }
        result["parity_sample"] = {"pairs": int(n_pairs), "max_abs": float(err.max()),
                                   "max_rel": float((err[big] / np.abs(want[big])).max()) if big.any() else 0.0}
    if nl == 1 and himpl == 0 and hidden_tokens > 0 and not args.no_next_rows:
        try:
            result["next_rows"] = {"absorbed_weight_hidden_path": absorbed_context(batch, layer, rn, args)}
        except Exception as exc:        # noqa: BLE001  (context beside the headline: never costs the line)
            result["next_rows"] = {"absorbed_weight_hidden_path": {"error": f"{type(exc).__name__}: {exc}"[:300]}}
    del rn, dls, layer
    torch.cuda.empty_cache()
    if sweep:
        result["sweep"] = sweep
        # Section 4.2, Eq. 6 models the extra time of hidden-cache requests as t = rho * m, linear in
        # their cached length: least-squares line of the item-kernel time over the hidden tokens
        x = np.array([p["hidden_tokens"] for p in sweep], dtype=np.float64)
        y = np.array([p["kernel_ms"] for p in sweep], dtype=np.float64)
        slope, icpt = np.polyfit(x, y, 1)
        resid = y - (slope * x + icpt)
        result["rho_fit"] = {"workload": cfg.name, "rho_us_per_hidden_token": slope * 1e3, "intercept_ms": icpt,
                             "r2": 1.0 - float((resid ** 2).sum() / ((y - y.mean()) ** 2).sum()),
                             "points": len(sweep)}
        if not args.no_next_rows and slope > 0:
            result.setdefault("next_rows", {})["schedule_with_fitted_rho"] = schedule_with_rho(batch, slope * 1e-3, args)
    if do_extras:
        others = {}
        for name, st, wu in (("opt13b", args.steps, args.warmup), ("opt30b", args.steps, args.warmup),
                             ("opt13b_step", max(2, args.steps // 5), 1)):
            # context beside the headline: a workload that cannot run here (say, not enough free HBM for the
            # 40 resident layers) is reported as such and never costs the line
            try:
                need = resident_bytes(wl.CONFIGS[name])
                free, _ = torch.cuda.mem_get_info()
                if need > 0.95 * free:
                    others[name] = {"skipped": f"needs {need / 2**30:.0f} GiB of HBM, {free / 2**30:.0f} GiB free"}
                    continue
                others[name] = dict(brief(measure(wl.CONFIGS[name], args, st, wu)), steps=st, warmup=wu)
            except Exception as exc:        # noqa: BLE001
                others[name] = {"error": f"{type(exc).__name__}: {exc}"[:300]}
                torch.cuda.empty_cache()
        result["other_configs"] = others
    print(json.dumps(result))


def schedule_with_rho(batch, rho_s_per_hidden_token, args):
    """The measured slope put to its use (Section 4.2, Eq. 6; Section 5, Definition 1): the requests of the bench
    batch as the candidates of one scheduling iteration.  m_i = the blocks of the request's KV cache (2 per
    block_size tokens), so a hidden-cache request of m_i costs rho * m_i with rho = slope * layers * block_size / 2;
    pending times are seeded exponential draws (mean 1 s: light load, mean 30 s: a long queue), the memory limit
    holds half of all the KV caches, |W| + |R| = batch."""
    import numpy as np
    from paper_2504_07494_amd import binding as ab
    cfg = batch.cfg
    mem = (2 * -(-batch.ctx_lens.astype(np.int64) // cfg.block_size)).astype(np.int64)
    limit = int(mem.sum() // 2)
    rho = rho_s_per_hidden_token * args.model_layers * cfg.block_size / 2.0
    rows = []
    for mean_s in (1.0, 30.0):
        pending = np.random.default_rng(cfg.seed).exponential(mean_s, size=batch.B)
        alpha, beta, val = ab.apt_schedule(pending, mem, limit, batch.B, rho)
        t = time.perf_counter()
        for _ in range(20):
            ab.apt_schedule(pending, mem, limit, batch.B, rho)
        ms = (time.perf_counter() - t) / 20 * 1e3
        order = np.argsort(-pending, kind="stable")      # longest-waiting first, KV cache only, until the memory is full
        fits = np.cumsum(mem[order]) <= limit
        kv_only = int(fits.sum()) if fits.all() else int(np.argmin(fits))
        rows.append({"mean_pending_s": mean_s, "scheduled": int(alpha.sum()),
                     "with_hidden_cache": int((alpha & beta).sum()),
                     "memory_used_blocks": int((mem * alpha * (1.0 - beta / 2.0)).sum()), "objective_s": val,
                     "kv_only_longest_waiting_first": {"scheduled": kv_only, "objective_s": float(pending[order[:kv_only]].sum())},
                     "ms_per_call": ms})
    return {"candidates": int(batch.B), "model_layers": args.model_layers, "rho_s_per_block_unit": rho,
            "memory_limit_blocks": limit, "cases": rows}


def run_sched_probe(args):
    """Section 6.6, scalability table: execution time of the scheduling algorithm against the number of
    candidate requests (the paper's numbers are from its implementation on its machine: context only).
    Candidates: contexts U[128, 2048] in blocks of 16, pending times Exp(1 s), memory for 40 % of the
    KV caches, rho as fitted by --sweep (per block of 16 tokens and request, 40 layers)."""
    import numpy as np
    from paper_2504_07494_amd import binding as ab
    paper_ms = {50: 0.3, 100: 0.5, 200: 1.0, 400: 2.1, 800: 4.8, 1600: 10.8}
    g = np.random.default_rng(2504)
    rho = 0.091e-6 * 16 * 40 / 2          # seconds per unit of m (m = 2 blocks per 16 tokens)
    rows = []
    for n, ref in paper_ms.items():
        mem = (2 * -(-g.integers(128, 2049, size=n) // 16)).astype(np.int64)
        pending = g.exponential(1.0, size=n)
        limit = int(mem.sum() * 0.4)
        ab.apt_schedule(pending, mem, limit, n, rho)
        reps = max(args.steps, 20)
        t = time.perf_counter()
        for _ in range(reps):
            alpha, beta, val = ab.apt_schedule(pending, mem, limit, n, rho)
        ms = (time.perf_counter() - t) / reps * 1e3
        rows.append({"candidates": n, "ms": ms, "paper_ms_other_machine": ref, "scheduled": int(alpha.sum()),
                     "hidden": int(beta.sum()), "value": val})
    print(json.dumps({"probe": "sched", "unit": "ms per apt_schedule call (host, one thread)", "rows": rows}))


def run_probe(args):
    """Calibration kernels of known work, for counter scaling and as context for the peaks."""
    import torch
    from paper_2504_07494_amd import binding as ab
    dev = torch.device("cuda:0")
    st = torch.cuda.current_stream(dev).cuda_stream
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if args.probe == "copy":
        n = 1 << 30
        src = torch.ones(n, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(args.warmup):
            ab.apt_copy_bytes(dst, src, n, st)
        a.record()
        for _ in range(args.steps):
            ab.apt_copy_bytes(dst, src, n, st)
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / args.steps
        print(json.dumps({"probe": "copy", "bytes_read": n, "bytes_written": n, "ms": ms,
                          "read_plus_write_GBs": 2 * n / ms / 1e6}))
    else:
        nwg, iters = 1024, 20000
        out = torch.empty(nwg * 256, dtype=torch.float32, device=dev)
        res = {"probe": "mfma"}
        for vname, variant, per_iter in (("f16_32x32x16", 0, 16 * 32768.0), ("f16_16x16x32", 1, 64 * 16384.0),
                                         ("bf16_32x32x16", 2, 16 * 32768.0), ("bf16_16x16x32", 3, 64 * 16384.0)):
            its = iters if per_iter < 1e6 else iters // 2
            flops = nwg * 4 * its * per_iter
            res[vname] = {"flops": flops}
            for name, rnd in (("constant_operands", 0), ("random_operands", 1)):
                for _ in range(args.warmup):
                    ab.apt_probe_mfma(out, nwg, its, rnd, variant, st)
                a.record()
                for _ in range(args.steps):
                    ab.apt_probe_mfma(out, nwg, its, rnd, variant, st)
                b.record()
                torch.cuda.synchronize()
                ms = a.elapsed_time(b) / args.steps
                res[vname][name] = {"ms": ms, "TFLOPs": flops / ms / 1e9}
        print(json.dumps(res))


if __name__ == "__main__":
    main()
