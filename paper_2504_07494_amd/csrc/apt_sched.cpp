// Greedy solution of the hybrid-cache scheduling problem (Section 5, Definition 1 and the
// marginal gains theta that follow it).  Host only.
#include <stdint.h>
#include <algorithm>
#include <vector>
#include "apt_internal.h"

namespace {
struct Cand {
    double theta;     // marginal gain in value per unit of memory
    int32_t r;        // request
    int32_t half;     // 0: first memory increment of the request, 1: second (hidden -> KV)
    int64_t dm;       // memory increment
    double gain;      // value increment
};
}  // namespace

extern "C" int apt_schedule(const double* pending, const int64_t* mem, int n, int64_t mem_limit, int32_t n_unfinished,
                            double rho, uint8_t* alpha, uint8_t* beta, double* value) {
    if (!pending || !mem || !alpha || !beta || n < 1 || mem_limit < 0 || n_unfinished < 0 || !(rho >= 0.0)) return APT_EINVAL;
    for (int i = 0; i < n; ++i)
        if (!(pending[i] >= 0.0) || mem[i] < 2 || (mem[i] & 1)) return APT_EINVAL;
    const double nrho = (double)n_unfinished * rho;
    // candidate schedules: per request either (0 -> m/2 as hidden cache, m/2 -> m as KV cache), or, when the
    // first of these gains less per unit of memory than going to KV cache directly, only (0 -> m)
    std::vector<Cand> cand;
    cand.reserve(2 * (size_t)n);
    for (int i = 0; i < n; ++i) {
        const double p = pending[i], m = (double)mem[i];
        const double th_hidden = 2.0 * p / m - 2.0 * nrho;
        const double th_kv = p / m;
        if (th_hidden < th_kv) {
            cand.push_back({th_kv, i, 0, mem[i], p});
        } else {
            cand.push_back({th_hidden, i, 0, mem[i] / 2, p - nrho * m});
            cand.push_back({2.0 * nrho, i, 1, mem[i] / 2, nrho * m});
        }
    }
    std::stable_sort(cand.begin(), cand.end(), [](const Cand& a, const Cand& b) {
        if (a.theta != b.theta) return a.theta > b.theta;
        if (a.r != b.r) return a.r < b.r;
        return a.half < b.half;
    });
    // greedy: best marginal gain first; a second increment needs its first; what does not fit is passed over
    std::vector<int64_t> used((size_t)n, 0);
    int64_t left = mem_limit;
    double total = 0.0;
    for (const Cand& c : cand) {
        if (c.half == 1 && used[c.r] != mem[c.r] / 2) continue;
        if (c.dm > left) continue;
        used[c.r] += c.dm;
        left -= c.dm;
        total += c.gain;
    }
    // the best single request alone (guards the approximation ratio against one large, valuable request)
    int best = -1, best_hidden = 0;
    double best_val = 0.0;
    for (int i = 0; i < n; ++i) {
        if (mem[i] <= mem_limit && pending[i] > best_val) { best = i; best_hidden = 0; best_val = pending[i]; }
        const double g = pending[i] - nrho * (double)mem[i];
        if (mem[i] / 2 <= mem_limit && g > best_val) { best = i; best_hidden = 1; best_val = g; }
    }
    if (best >= 0 && best_val > total) {
        for (int i = 0; i < n; ++i) alpha[i] = beta[i] = 0;
        alpha[best] = 1;
        beta[best] = (uint8_t)best_hidden;
        total = best_val;
    } else {
        for (int i = 0; i < n; ++i) {
            alpha[i] = used[i] > 0;
            beta[i] = used[i] > 0 && used[i] < mem[i];
        }
    }
    if (value) *value = total;
    return APT_OK;
}
