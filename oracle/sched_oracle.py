"""Test infrastructure: the hybrid-cache scheduling problem (Section 5, Definition 1) by its
definition, and the greedy solution described after it.  Only tests and bench.py's reference
leg may import this module.

Definition 1: choose alpha_i, beta_i in {0, 1} for the candidates i to maximise sum g_i alpha_i with
g_i = p_i - beta_i (|W| + |R|) rho m_i, subject to sum (1 - beta_i / 2) m_i alpha_i <= M."""
import itertools


def value_and_memory(pending, mem, n_unfinished, rho, alpha, beta):
    val = sum(a * (p - b * n_unfinished * rho * m) for p, m, a, b in zip(pending, mem, alpha, beta))
    used = sum(a * (m - b * m // 2) for m, a, b in zip(mem, alpha, beta))
    return val, used


def optimum(pending, mem, mem_limit, n_unfinished, rho):
    """Exhaustive search over (not scheduled, KV cache, hidden cache) per request: tiny inputs only."""
    best = 0.0
    for choice in itertools.product((0, 1, 2), repeat=len(pending)):
        alpha = [c > 0 for c in choice]
        beta = [c == 2 for c in choice]
        val, used = value_and_memory(pending, mem, n_unfinished, rho, alpha, beta)
        if used <= mem_limit and val > best:
            best = val
    return best


def greedy(pending, mem, mem_limit, n_unfinished, rho):
    """Marginal gains theta per unit of memory as given after Definition 1: from 0 to m/2 (hidden
    cache) 2p/m - 2(|W|+|R|)rho, from m/2 to m (KV cache) 2(|W|+|R|)rho; if the first is smaller
    than p/m, the gain of going to KV cache directly, hidden cache is not offered for that request.
    Candidates are taken by decreasing theta (ties: request index, then first increment first) while
    they fit; the result is compared with the best single request.  Returns (alpha, beta, value)."""
    n = len(pending)
    nrho = n_unfinished * rho
    cand = []
    for i in range(n):
        p, m = pending[i], float(mem[i])
        th_hidden, th_kv = 2.0 * p / m - 2.0 * nrho, p / m
        if th_hidden < th_kv:
            cand.append((th_kv, i, 0, mem[i], p))
        else:
            cand.append((th_hidden, i, 0, mem[i] // 2, p - nrho * m))
            cand.append((2.0 * nrho, i, 1, mem[i] // 2, nrho * m))
    cand.sort(key=lambda c: (-c[0], c[1], c[2]))
    used, left, total = [0] * n, mem_limit, 0.0
    for theta, r, half, dm, gain in cand:
        if half == 1 and used[r] != mem[r] // 2:
            continue
        if dm > left:
            continue
        used[r] += dm
        left -= dm
        total += gain
    best, best_hidden, best_val = -1, 0, 0.0
    for i in range(n):
        if mem[i] <= mem_limit and pending[i] > best_val:
            best, best_hidden, best_val = i, 0, pending[i]
        g = pending[i] - nrho * float(mem[i])
        if mem[i] // 2 <= mem_limit and g > best_val:
            best, best_hidden, best_val = i, 1, g
    if best >= 0 and best_val > total:
        alpha = [int(i == best) for i in range(n)]
        beta = [int(i == best and best_hidden) for i in range(n)]
        return alpha, beta, best_val
    return [int(u > 0) for u in used], [int(0 < u < m) for u, m in zip(used, mem)], total
