#!/usr/bin/env python3
"""Benchmark of the hybrid-cache decode attention step on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W [--config opt13b] [--hidden-ratio R]

A step is one pass of the whole hot path for one layer over one synthetic batch whose
inputs are already resident in HBM: the ragged work partition (host planner + copy of the
plan to the device), the item kernel (paged-KV attention and hidden-cache recompute +
attention in one launch) and the merge kernel.  The metric is cached tokens per second
per decode layer = sum of the batch's context lengths / time per step.

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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="opt13b")
    ap.add_argument("--hidden-ratio", type=float, default=None)
    ap.add_argument("--kv-chunk", type=int, default=0)
    ap.add_argument("--hidden-impl", choices=["auto", "valu", "mfma", "absorbed"], default="auto",
                    help="hidden-kind kernel; 'absorbed' is the re-associated form without K/V projection (its "
                         "roofline entry is priced on its own work, never against the MFMA target)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-next-rows", action="store_true",
                    help="skip the short extra measurement of the absorbed-weight hidden path (single-layer runs "
                         "of the default hidden path add it under 'next_rows'; it never enters 'value')")
    ap.add_argument("--pairs-per-thread", type=int, default=48)
    ap.add_argument("--sweep", action="store_true",
                    help="also time hidden-cache ratios 0/25/50/75/100 %% of the same config (adds a 'sweep' list)")
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

    cfg = wl.CONFIGS[args.config]
    if args.hidden_ratio is not None:
        cfg = wl.with_ratio(cfg, args.hidden_ratio)
    t_gen = time.time()
    batch = wl.make_batch(cfg)
    nl = cfg.n_layers
    himpl = {"auto": 0, "valu": 1, "mfma": 2, "absorbed": 3}[args.hidden_impl]
    rn = DecodeRunner(batch, kv_chunk=args.kv_chunk, hidden_impl=himpl)
    layer, dls = None, []
    for li in range(nl):                      # every layer of the step is resident in HBM
        layer = wl.make_layer(batch, layer=li, workers=min(16, os.cpu_count() or 8))
        dls.append(rn.upload(layer, keep_raw_weights=(nl == 1 or himpl == 3)))
    t_gen = time.time() - t_gen
    dl = dls[-1]                              # `layer` is its host copy (cpu_baseline / parity sample)
    torch.cuda.synchronize()

    for _ in range(args.warmup):
        rn.run_step(dls)
    torch.cuda.synchronize()

    ev = HipEvents(args.steps * nl)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        rn.plan()
        for li in range(nl):
            rn.run(dls[li], ev.pairs[i * nl + li][0], ev.pairs[i * nl + li][1])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kern_ms = [ev.elapsed_ms(i) for i in range(args.steps * nl)]
    ev.close()
    kern_avg_ms = float(np.mean(kern_ms))

    total_tokens = batch.total_tokens
    hidden_tokens = batch.hidden_tokens
    kv_tokens = batch.kv_tokens
    d, e = cfg.d_model, wl.ELEM_BYTES[cfg.dtype]
    # cached tokens per second per decode layer: a step of nl layers serves total_tokens in each layer
    value = total_tokens * nl / (ms_per_step * 1e-3)

    # algorithmic work of the item kernel per launch
    flops = 4.0 * d * d * hidden_tokens                 # K and V projections of hidden-kind tokens
    kv_bytes = 2.0 * d * e * kv_tokens                  # K row + V row of KV-kind tokens
    hid_bytes = 1.0 * d * e * hidden_tokens
    t_mfma = flops / (PEAK_MFMA_TFLOPS[cfg.dtype] * 1e12)
    t_hbm = (kv_bytes + hid_bytes) / (PEAK_HBM_GBS * 1e9)
    wkey = f"{cfg.name}@{cfg.hidden_ratio:g}"
    if rn.info.hidden_impl == 3 and hidden_tokens > 0:
        # absorbed form: no projection; per hidden token and head one d_model-long dot product and one
        # d_model-long weighted row update (4 d H flops, on the matrix cores with the fp32 operand split
        # into 16-bit parts); the hidden rows are read twice.  Priced against HBM, on its own bytes.
        flops = 4.0 * d * cfg.n_heads * hidden_tokens
        hid_bytes = 2.0 * d * e * hidden_tokens
        ach = (kv_bytes + hid_bytes) / (kern_avg_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": ach / PEAK_HBM_GBS, "traffic": read_traffic(wkey + "@absorbed")}
    elif t_mfma >= t_hbm:
        ach = flops / (kern_avg_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": PEAK_MFMA_TFLOPS[cfg.dtype], "unit": "TFLOP/s",
                "frac": ach / PEAK_MFMA_TFLOPS[cfg.dtype], "traffic": read_traffic(wkey)}
    else:
        ach = (kv_bytes + hid_bytes) / (kern_avg_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": ach / PEAK_HBM_GBS, "traffic": read_traffic(wkey)}
    mfma_items = rn.info.n_hidden_items > 0 and rn.info.hidden_impl == 2
    kname = "apt_items_mfma_kernel" if mfma_items else "apt_items_kernel"
    if rn.info.hidden_impl == 3 and hidden_tokens > 0:
        kname = "apt_absorb_{q,score,stats,pv,out,final}_kernel + apt_items_kernel (one event pair around all seven)"
    roof.update({"kernel": kname, "kernel_ms": kern_avg_ms, "kernel_ms_min": float(np.min(kern_ms)),
                 "algorithmic_flops": flops, "algorithmic_bytes": kv_bytes + hid_bytes})

    result = {
        "metric": "cached tokens/sec per decode layer; HBM GB/s and MFMA util vs MI355X peak",
        "value": value, "unit": "cached tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: d_model={d}, {cfg.n_heads} heads x {cfg.head_dim}, {cfg.dtype}, "
                               f"batch {batch.B}, ctx {cfg.len_dist}[{cfg.len_lo},{cfg.len_hi}], block {cfg.block_size}, "
                               f"{int(round(100 * cfg.hidden_ratio))}% hidden-cache requests"
                               + (f", {nl} layers per step (one plan, {nl} attention calls)" if nl > 1 else ""),
                   "layers_per_step": nl,
                   "total_tokens": total_tokens, "hidden_tokens": hidden_tokens, "kv_tokens": kv_tokens,
                   "hidden_impl": {1: "valu", 2: "mfma", 3: "absorbed"}[int(rn.info.hidden_impl)],
                   "n_items": int(rn.info.n_items), "n_hidden_items": int(rn.info.n_hidden_items),
                   "seed": cfg.seed, "input_gen_s": round(t_gen, 2)},
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
    if nl == 1 and himpl == 0 and hidden_tokens > 0 and not args.no_next_rows and not args.sweep:
        # context only: the same step with hidden-kind requests through the absorbed-weight form (no K/V
        # projection: not the paper's method, so it is never the headline and never priced in projection flops)
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
        result["next_rows"] = {"absorbed_weight_hidden_path": {
            "ms_per_step": ms2, "cached_tokens_per_s": total_tokens / (ms2 * 1e-3),
            "max_abs_difference_to_default_path": dev,
            "hbm_frac_on_own_bytes": (kv_bytes + 2.0 * d * e * hidden_tokens) / (ms2 * 1e-3) / 1e9 / PEAK_HBM_GBS}}
        del rn2, dl2
    if args.sweep:
        del rn, dls, dl
        torch.cuda.empty_cache()
        sweep = [time_ratio(cfg, r, args) for r in (0.0, 0.25, 0.5, 0.75, 1.0)]
        result["sweep"] = sweep
        # Section 4.2, Eq. 6 models the extra time of hidden-cache requests as t = rho * m, linear in
        # their cached length: least-squares line of the item-kernel time over the hidden tokens
        x = np.array([p["hidden_tokens"] for p in sweep], dtype=np.float64)
        y = np.array([p["kernel_ms"] for p in sweep], dtype=np.float64)
        slope, icpt = np.polyfit(x, y, 1)
        resid = y - (slope * x + icpt)
        result["rho_fit"] = {"rho_us_per_hidden_token": slope * 1e3, "intercept_ms": icpt,
                             "r2": 1.0 - float((resid ** 2).sum() / ((y - y.mean()) ** 2).sum())}
    print(json.dumps(result))


def time_ratio(cfg, ratio, args):
    """Item-kernel time and roofline fractions of one hidden-cache ratio (same lengths, nested kind sets)."""
    import numpy as np
    import torch
    from paper_2504_07494_amd import workloads as wl
    from paper_2504_07494_amd.harness import DecodeRunner
    c = wl.with_ratio(cfg, ratio)
    batch = wl.make_batch(c)
    layer = wl.make_layer(batch, workers=min(16, os.cpu_count() or 8))
    rn = DecodeRunner(batch, kv_chunk=args.kv_chunk,
                      hidden_impl={"auto": 0, "valu": 1, "mfma": 2, "absorbed": 3}[args.hidden_impl])
    dl = rn.upload(layer)
    for _ in range(args.warmup):
        rn.plan()
        rn.run(dl)
    torch.cuda.synchronize()
    ev = HipEvents(args.steps)
    t0 = time.perf_counter()
    for i in range(args.steps):
        rn.plan()
        rn.run(dl, ev.pairs[i][0], ev.pairs[i][1])
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / args.steps
    kms = float(np.mean([ev.elapsed_ms(i) for i in range(args.steps)]))
    ev.close()
    d, e = c.d_model, wl.ELEM_BYTES[c.dtype]
    absorbed = int(rn.info.hidden_impl) == 3
    flops = 4.0 * d * d * batch.hidden_tokens
    nbytes = 2.0 * d * e * batch.kv_tokens + (2.0 if absorbed else 1.0) * d * e * batch.hidden_tokens
    del rn, dl, layer
    torch.cuda.empty_cache()
    row = {"hidden_ratio": ratio, "total_tokens": batch.total_tokens, "hidden_tokens": batch.hidden_tokens,
           "ms_per_step": ms_step, "kernel_ms": kms, "cached_tokens_per_s": batch.total_tokens / (ms_step * 1e-3),
           "hbm_gbs": nbytes / (kms * 1e-3) / 1e9, "hbm_frac": nbytes / (kms * 1e-3) / 1e9 / PEAK_HBM_GBS}
    if not absorbed:        # the absorbed form does no projection: it is never priced in projection flops
        row.update({"mfma_tflops": flops / (kms * 1e-3) / 1e12,
                    "mfma_frac": flops / (kms * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS[c.dtype]})
    return row


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
        res = {"probe": "mfma", "flops": nwg * 4 * iters * 16 * 32768.0}
        for name, rnd in (("constant_operands", 0), ("random_operands", 1)):
            for _ in range(args.warmup):
                ab.apt_probe_mfma(out, nwg, iters, rnd, st)
            a.record()
            for _ in range(args.steps):
                ab.apt_probe_mfma(out, nwg, iters, rnd, st)
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b) / args.steps
            res[name] = {"ms": ms, "TFLOPs": res["flops"] / ms / 1e9}
        print(json.dumps(res))


if __name__ == "__main__":
    main()
