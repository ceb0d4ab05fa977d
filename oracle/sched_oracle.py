"""Test infrastructure: the hybrid-cache scheduling problem (Section 5, Definition 1) by its
definition, and the greedy solution described after it (restated from the paper's wording, state by
state; it shares no structure with the library's sorted-candidate implementation).  Only tests and bench.py's reference
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


def theta(p, m, used, nrho):
    """Marginal gain in value per unit of memory of request (p, m) at its current memory usage `used`
    (the two case tables after Definition 1).  Returns (theta, memory increment) or None when the
    request already holds its KV cache.  From 0 the request is offered its hidden cache (half the
    memory) unless that gains less per unit than taking the KV cache at once."""
    if used == 0:
        to_hidden = 2 * p / m - 2 * nrho      # (p - nrho m - 0) / (m/2 - 0), in the simplified form the paper prints
        to_kv = p / m                         # (p - 0) / (m - 0)
        return (to_hidden, m // 2) if to_hidden >= to_kv else (to_kv, m)
    if 2 * used == m:
        return 2 * nrho, m // 2               # (p - (p - nrho m)) / (m - m/2): the same for every request
    return None


def greedy(pending, mem, mem_limit, n_unfinished, rho):
    """The greedy process in the paper's own terms: every request has a current memory usage (0, m/2
    or m); over and over, the request whose marginal gain theta at its CURRENT usage is largest
    (ties: lowest request index) among those whose memory increment still fits gets that increment.
    Nothing is precomputed or sorted.  The final usage gives the schedule: 0 = not scheduled, m/2 =
    hidden cache, m = KV cache.  As in every density greedy with a factor-2 guarantee, the result is
    then compared with the best schedule that serves a single request (evaluated with Definition 1
    itself).  Returns (alpha, beta, value)."""
    n = len(pending)
    nrho = n_unfinished * rho
    used = [0] * n
    left = mem_limit
    while True:
        pick = None
        for i in range(n):
            move = theta(pending[i], mem[i], used[i], nrho)
            if move is None or move[1] > left:
                continue
            if pick is None or move[0] > pick[0]:
                pick = (move[0], i, move[1])
        if pick is None:
            break
        used[pick[1]] += pick[2]
        left -= pick[2]
    alpha = [int(u > 0) for u in used]
    beta = [int(0 < u < m) for u, m in zip(used, mem)]
    val, _ = value_and_memory(pending, mem, n_unfinished, rho, alpha, beta)
    for i in range(n):
        for hidden in (0, 1):
            a1 = [int(j == i) for j in range(n)]
            b1 = [int(j == i and hidden) for j in range(n)]
            v1, m1 = value_and_memory(pending, mem, n_unfinished, rho, a1, b1)
            if m1 <= mem_limit and v1 > val:
                alpha, beta, val = a1, b1, v1
    return alpha, beta, val
