"""Greedy solution of the hybrid-cache scheduling problem (Section 5, Definition 1).  The rule
(oracle/sched_oracle.greedy: the paper's state-by-state marginal-gain process, written without a
candidate list or a sort) is pinned against the problem's definition by exhaustive search on tiny
instances (feasible, and at least half of the optimum) and by cases whose answer is known.  The C
ABI is checked the same way against Definition 1 directly (feasible, >= half of the exhaustive
optimum, objective equals the definition's value of its decisions, invariance under rescaling of
time), and decision by decision against the rule."""
import time

import numpy as np
import pytest

from oracle import sched_oracle as so
from paper_2504_07494_amd import binding as ab


def _instance(g, n, tight):
    mem = (2 * g.integers(1, 129, size=n)).astype(np.int64)              # KV blocks of contexts up to 2048 tokens (16 per block)
    pending = np.round(g.exponential(1.0, size=n) * 1000) / 1000         # seconds
    limit = int(mem.sum() * tight)
    return pending.astype(np.float64), mem, limit


@pytest.mark.parametrize("seed", range(6))
def test_rule_is_feasible_and_within_a_factor_two_of_the_exhaustive_optimum(seed):
    g = np.random.default_rng(seed)
    for _ in range(40):
        n = int(g.integers(1, 8))
        pending, mem, limit = _instance(g, n, g.choice([0.1, 0.3, 0.5, 0.8, 1.2]))
        n_unf, rho = int(g.integers(1, 60)), float(g.choice([0.0, 1e-5, 1e-4, 1e-3, 1e-2]))
        alpha, beta, val = so.greedy(pending.tolist(), mem.tolist(), limit, n_unf, rho)
        got_val, used = so.value_and_memory(pending, mem, n_unf, rho, alpha, beta)
        assert used <= limit and abs(got_val - val) <= 1e-9 * max(1.0, abs(val))
        assert all(b <= a for a, b in zip(alpha, beta))
        opt = so.optimum(pending.tolist(), mem.tolist(), limit, n_unf, rho)
        assert val >= 0.5 * opt - 1e-12 and val <= opt + 1e-9, (val, opt)


def test_known_cases():
    pending, mem = [3.0, 1.0, 2.0, 0.5], [40, 10, 60, 20]
    # plenty of memory: everyone is scheduled with KV cache (the second increment still gains value)
    a, b, v = so.greedy(pending, mem, 130, 4, 1e-3)
    assert a == [1, 1, 1, 1] and b == [0, 0, 0, 0] and abs(v - 6.5) < 1e-12
    # no latency penalty (rho = 0): half the memory suffices for the full value, with hidden cache
    a, b, v = so.greedy(pending, mem, 65, 4, 0.0)
    assert a == [1, 1, 1, 1] and b == [1, 1, 1, 1] and abs(v - 6.5) < 1e-12
    # a penalty so large that hidden cache never pays: plain knapsack by value density, KV cache only
    a, b, v = so.greedy(pending, mem, 60, 4, 10.0)
    assert b == [0, 0, 0, 0] and a == [1, 1, 0, 0] and abs(v - 4.0) < 1e-12
    # memory-tight: hidden cache lets more requests in than KV cache alone would
    a, b, v = so.greedy(pending, mem, 70, 4, 1e-4)
    assert sum(a) == 4 and sum(b) >= 3
    # one request that fits only with hidden cache
    a, b, v = so.greedy([2.0], [100], 50, 1, 1e-3)
    assert a == [1] and b == [1] and abs(v - (2.0 - 1e-3 * 100)) < 1e-12
    # nothing fits
    assert so.greedy([2.0], [100], 49, 1, 1e-3) == ([0], [0], 0.0)
    # the single valuable request beats the dense small ones: density order alone would take request 0 first
    a, b, v = so.greedy([1.0, 50.0], [2, 200], 200, 2, 10.0)
    assert a == [0, 1] and b == [0, 0] and v == 50.0


@pytest.mark.parametrize("seed", range(4))
def test_c_abi_against_definition_1_directly(seed):
    g = np.random.default_rng(50 + seed)
    for _ in range(40):
        n = int(g.integers(1, 8))
        pending, mem, limit = _instance(g, n, g.choice([0.1, 0.3, 0.5, 0.8, 1.2]))
        n_unf, rho = int(g.integers(1, 60)), float(g.choice([0.0, 1e-5, 1e-4, 1e-3, 1e-2]))
        alpha, beta, val = ab.apt_schedule(pending, mem, limit, n_unf, rho)
        got_val, used = so.value_and_memory(pending, mem, n_unf, rho, alpha.tolist(), beta.tolist())
        assert used <= limit and all(b <= a for a, b in zip(alpha, beta))
        assert abs(got_val - val) <= 1e-9 * max(1.0, abs(val))
        opt = so.optimum(pending.tolist(), mem.tolist(), limit, n_unf, rho)
        assert 0.5 * opt - 1e-12 <= val <= opt + 1e-9, (val, opt)
        # time measured in another unit (pending times and rho scaled by a power of two): same decisions
        a2, b2, v2 = ab.apt_schedule(pending * 4.0, mem, limit, n_unf, rho * 4.0)
        assert a2.tolist() == alpha.tolist() and b2.tolist() == beta.tolist() and abs(v2 - 4.0 * val) <= 1e-9 * max(1.0, v2)


@pytest.mark.parametrize("seed,n", [(0, 1), (1, 7), (2, 50), (3, 400), (4, 1600)])
def test_c_abi_takes_the_same_decisions_as_the_rule(seed, n):
    g = np.random.default_rng(100 + seed)
    for tight in (0.05, 0.4, 0.9, 1.5):
        pending, mem, limit = _instance(g, n, tight)
        n_unf, rho = n + int(g.integers(0, 50)), float(g.choice([0.0, 2e-6, 1e-4, 5e-3]))
        alpha, beta, val = ab.apt_schedule(pending, mem, limit, n_unf, rho)
        wa, wb, wv = so.greedy(pending.tolist(), mem.tolist(), limit, n_unf, rho)
        assert alpha.tolist() == wa and beta.tolist() == wb
        assert abs(val - wv) <= 1e-9 * max(1.0, abs(wv))


def test_c_abi_rejects_bad_arguments_and_is_fast_enough():
    p, m = np.array([1.0, 2.0]), np.array([4, 6], dtype=np.int64)
    for bad in (lambda: ab.apt_schedule(p, np.array([4, 5], dtype=np.int64), 10, 2, 0.1),      # odd memory
                lambda: ab.apt_schedule(np.array([1.0, -1.0]), m, 10, 2, 0.1),
                lambda: ab.apt_schedule(p, m, -1, 2, 0.1), lambda: ab.apt_schedule(p, m, 10, 2, -0.1),
                lambda: ab.apt_schedule(p, m, 10, 2, float("nan"))):
        with pytest.raises(ab.AptError) as e:
            bad()
        assert e.value.status == ab.APT_EINVAL
    # Table 6 of the paper reports 10.8 ms for 1600 candidate requests (its implementation, its machine)
    g = np.random.default_rng(5)
    pending, mem, limit = _instance(g, 1600, 0.4)
    ab.apt_schedule(pending, mem, limit, 1600, 1e-4)
    t = time.perf_counter()
    for _ in range(20):
        ab.apt_schedule(pending, mem, limit, 1600, 1e-4)
    ms = (time.perf_counter() - t) / 20 * 1e3
    print(f"apt_schedule, 1600 candidates: {ms:.3f} ms")
    assert ms < 10.8


def test_schedule_and_pool_compose_admitted_requests_always_fit_and_can_grow():
    """Prefill iterations of a small serving simulation: the candidates are the waiting requests, the
    memory constraint is the pool size minus the maximum requirement of the running requests
    (Section 5, after Definition 1), m_i is a request's KV blocks at its maximum length.  Whatever the
    greedy schedule admits can then be assigned in the pool in the kind it chose and extended to its
    maximum length without ever running out of blocks."""
    g = np.random.default_rng(9)
    n_blocks, bs, mb, nslots = 400, 16, 16, 24
    pool = ab.apt_pool_create(n_blocks, bs, mb, nslots)
    waiting, running, t = [], {}, 0.0            # waiting: (arrival time, prompt, max_len); running: slot -> dict
    rho = 2e-4
    admitted_hidden = admitted_kv = 0
    try:
        for it in range(300):
            t += 0.05
            for _ in range(g.poisson(0.7)):
                prompt = int(g.integers(1, 120))
                waiting.append((t, prompt, min(mb * bs, prompt + int(g.integers(1, 120)))))
            # decode progress and departures
            for slot in list(running):
                r = running[slot]
                if r["len"] < r["max_len"]:
                    r["len"] += 1
                    ab.apt_pool_extend(pool, slot, r["len"])      # never APT_EFULL: the growth was reserved
                else:
                    ab.apt_pool_release(pool, slot)
                    del running[slot]
            free_slots = [s for s in range(nslots) if s not in running]
            if not waiting or not free_slots:
                continue
            cand = waiting[:len(free_slots)]
            pending = np.array([t - a for a, _, _ in cand], dtype=np.float64)
            mem = np.array([2 * -(-m // bs) for _, _, m in cand], dtype=np.int64)
            reserved = sum((2 if r["kind"] == 0 else 1) * -(-r["max_len"] // bs) for r in running.values())
            limit = n_blocks - reserved
            alpha, beta, _ = ab.apt_schedule(pending, mem, max(limit, 0), len(waiting) + len(running), rho)
            used = sum(int(m) // (2 if b else 1) for m, a, b in zip(mem, alpha, beta) if a)
            assert used <= max(limit, 0)
            keep = []
            for (arr, prompt, max_len), a, b in zip(cand, alpha, beta):
                if not a:
                    keep.append((arr, prompt, max_len))
                    continue
                slot = free_slots.pop(0)
                kind = 1 if b else 0
                ab.apt_pool_assign(pool, slot, kind, prompt)       # never APT_EFULL
                running[slot] = {"kind": kind, "len": prompt, "max_len": max_len}
                admitted_hidden += int(b)
                admitted_kv += int(not b)
            waiting = keep + waiting[len(cand):]
            assert ab.apt_pool_free_blocks(pool) >= 0
        assert admitted_hidden > 0 and admitted_kv > 0          # the simulation exercised both cache kinds
    finally:
        ab.apt_pool_destroy(pool)


def test_bench_scheduling_example_is_feasible_and_uses_hidden_caches_only_when_waiting_outweighs_recompute():
    """bench.py's use of the fitted slope (Section 4.2, Eq. 6 into Definition 1): host only."""
    import types
    import bench
    from paper_2504_07494_amd import workloads as wl
    batch = wl.make_batch(wl.CONFIGS["opt66b"])
    out = bench.schedule_with_rho(batch, 0.27e-6, types.SimpleNamespace(model_layers=64))
    light, queue = out["cases"]
    for c in (light, queue):
        assert c["memory_used_blocks"] <= out["memory_limit_blocks"]
        assert c["objective_s"] >= c["kv_only_longest_waiting_first"]["objective_s"] * 0.5     # the rule's guarantee
        assert c["scheduled"] >= c["kv_only_longest_waiting_first"]["scheduled"]
    assert light["with_hidden_cache"] == 0 and queue["with_hidden_cache"] > 0
    # a free recompute (rho = 0) puts every scheduled request on the hidden cache and fits them all in half the memory
    free = bench.schedule_with_rho(batch, 0.0, types.SimpleNamespace(model_layers=64))["cases"][0]
    assert free["scheduled"] == free["with_hidden_cache"] == batch.B
