"""Greedy solution of the hybrid-cache scheduling problem (Section 5, Definition 1).  The rule is
pinned against the problem's definition by exhaustive search on tiny instances (feasible, and at
least half of the optimum) and by cases whose answer is known; the C ABI is compared with the
rule decision by decision."""
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
