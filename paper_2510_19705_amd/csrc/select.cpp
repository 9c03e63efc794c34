// Host-side latency model and hierarchy selection (Sec. 3.3 Thm 3.2, Sec. 4.1 Cor. 4.1, Sec. 4.2-4.3).
//
// gamma(alpha, T_i, T_j) is evaluated exactly from its definition (expected number of draft+verify
// rounds until T_j tokens are collected when each round offers T_i drafts and yields the accepted
// ones plus one) instead of being estimated by simulation as in the paper.  The minimisation over
// hierarchies walks the reduction graph of Sec. 4.3 directly: apart from the zero-cost self-loops
// at the (M_i, L) vertices the graph is acyclic (edges go from (M_i, j) to (M_k, l) with k < i), so
// the cheapest augmented path is a bottom-up dynamic programme over the vertices (M_i, j); edge
// multipliers and costs are those of the paper's edge table.
#include <math.h>
#include <stdarg.h>

#include <map>
#include <vector>

#include "../../include/hsd.h"

void hsd_set_error(const char* fmt, ...);

namespace {

double top_factor(double a, int T) {          // (1 - a) / (1 - a^(T+1)) = 1 / sum_{i<=T} a^i
    double s = 0.0, p = 1.0;
    for (int i = 0; i <= T; ++i) { s += p; p *= a; }
    return 1.0 / s;
}

// P(n drafts accepted out of t): a^n (1-a) for n < t, a^t for n = t
void accepted_pmf(double a, int t, std::vector<double>& pmf) {
    pmf.assign(t + 1, 0.0);
    double p = 1.0;
    for (int n = 0; n < t; ++n) { pmf[n] = p * (1.0 - a); p *= a; }
    pmf[t] = p;
}

double gamma_rounds(double a, int Ti, int Tj) {
    std::vector<double> pmf;
    accepted_pmf(a, Ti, pmf);
    std::vector<double> E(Tj + Ti + 2, 0.0);      // E[c]: expected further rounds holding c tokens
    for (int c = Tj - 1; c >= 0; --c) {
        double e = 1.0;
        for (int n = 0; n <= Ti; ++n) e += pmf[n] * E[c + n + 1];
        E[c] = e;
    }
    return E[0];
}

bool valid_rate(double a) { return a >= 0.0 && a <= 1.0; }

double latency_literal(int n, const double* c, const double* a, const int* T) {
    const int K = n - 1;
    if (K == 0) return c[0];
    double inner = T[0] * c[0];
    for (int i = 1; i < K; ++i) inner = gamma_rounds(a[i - 1], T[i - 1], T[i]) * (c[i] + inner);
    return top_factor(a[K - 1], T[K - 1]) * (c[K] + inner);
}

double latency_overshoot(int n, const double* c, const double* a, const int* T) {
    const int K = n - 1;
    if (K == 0) return c[0];
    std::map<int, double> batch;                  // law of the batch length handed up
    batch[T[0]] = 1.0;
    double cost = T[0] * c[0];
    std::vector<double> pmf;
    for (int idx = 1; idx < K; ++idx) {
        const int need = T[idx];
        std::map<int, double> gain;               // tokens gained per round = accepted + 1
        for (auto& b : batch) {
            accepted_pmf(a[idx - 1], b.first, pmf);
            for (int k = 0; k <= b.first; ++k) gain[k + 1] += b.second * pmf[k];
        }
        std::vector<double> rounds(need, 0.0);
        std::vector<std::map<int, double>> fin(need);
        for (int cnt = need - 1; cnt >= 0; --cnt) {
            double r = 1.0;
            for (auto& g : gain) {
                const int nxt = cnt + g.first;
                if (nxt >= need) fin[cnt][nxt] += g.second;
                else {
                    r += g.second * rounds[nxt];
                    for (auto& f : fin[nxt]) fin[cnt][f.first] += g.second * f.second;
                }
            }
            rounds[cnt] = r;
        }
        cost = rounds[0] * (cost + c[idx]);
        batch = fin[0];
    }
    double tokens = 0.0;
    for (auto& b : batch) tokens += b.second / top_factor(a[K - 1], b.first);
    return (cost + c[K]) / tokens;
}

}  // namespace

extern "C" double hsd_gamma(double alpha, int Ti, int Tj) {
    if (!valid_rate(alpha) || Ti < 1 || Tj < 1) return -1.0;
    return gamma_rounds(alpha, Ti, Tj);
}

extern "C" double hsd_expected_latency(int n, const double* cost, const double* alpha_adj, const int* T, int exact_overshoot) {
    if (n < 1 || !cost || (n > 1 && (!alpha_adj || !T))) return -1.0;
    for (int i = 0; i < n; ++i)
        if (!(cost[i] > 0.0)) return -1.0;
    for (int i = 0; i + 1 < n; ++i)
        if (!valid_rate(alpha_adj[i]) || T[i] < 1) return -1.0;
    return exact_overshoot ? latency_overshoot(n, cost, alpha_adj, T) : latency_literal(n, cost, alpha_adj, T);
}

extern "C" int hsd_select_hierarchy(int n_models, const double* cost, const double* alpha, int Tbar, int monotone_T,
                                    int* sigma_out, int* T_out, int* n_sigma, double* latency_out) {
    if (n_models < 1 || !cost || !alpha || Tbar < 1 || !sigma_out || !T_out || !n_sigma || !latency_out) {
        hsd_set_error("hsd_select_hierarchy: bad arguments");
        return HSD_EINVAL;
    }
    const int K = n_models - 1;
    for (int i = 0; i <= K; ++i) {
        if (!(cost[i] > 0.0)) { hsd_set_error("hsd_select_hierarchy: cost[%d] must be positive", i); return HSD_EINVAL; }
        for (int j = i + 1; j <= K; ++j)
            if (!valid_rate(alpha[i * n_models + j])) { hsd_set_error("hsd_select_hierarchy: alpha[%d][%d] outside [0,1]", i, j); return HSD_EINVAL; }
    }
    // g[i][j]: cheapest expected cost of one batch from vertex (M_i, j); below[i][j]: the vertex it draws from
    std::vector<double> g((size_t)K * (Tbar + 1), 0.0);
    std::vector<int> below_m((size_t)K * (Tbar + 1), -1), below_t((size_t)K * (Tbar + 1), 0);
    auto at = [&](int i, int j) { return (size_t)i * (Tbar + 1) + j; };
    for (int i = 0; i < K; ++i)
        for (int j = 1; j <= Tbar; ++j) {
            double best = j * cost[i];            // edge to (M_i, L): M_i drafts j tokens itself
            int bm = -1, bt = 0;
            for (int k = 0; k < i; ++k)
                for (int l = 1; l <= (monotone_T ? j : Tbar); ++l) {
                    const double v = gamma_rounds(alpha[k * n_models + i], l, j) * (cost[i] + g[at(k, l)]);
                    if (v < best) { best = v; bm = k; bt = l; }
                }
            g[at(i, j)] = best;
            below_m[at(i, j)] = bm;
            below_t[at(i, j)] = bt;
        }
    double best = cost[K];
    int bm = -1, bt = 0;
    for (int i = 0; i < K; ++i)
        for (int j = 1; j <= Tbar; ++j) {
            const double v = top_factor(alpha[i * n_models + K], j) * (cost[K] + g[at(i, j)]);
            if (v < best) { best = v; bm = i; bt = j; }
        }
    std::vector<int> sig, Ts;
    sig.push_back(K);
    while (bm >= 0) {
        sig.push_back(bm);
        Ts.push_back(bt);
        const size_t a = at(bm, bt);
        bm = below_m[a];
        bt = below_t[a];
    }
    *n_sigma = (int)sig.size();
    for (size_t i = 0; i < sig.size(); ++i) sigma_out[i] = sig[sig.size() - 1 - i];
    for (size_t i = 0; i < Ts.size(); ++i) T_out[i] = Ts[Ts.size() - 1 - i];
    *latency_out = best;
    return HSD_OK;
}

extern "C" int hsd_best_single_draft(int n_models, const double* cost, const double* alpha, int Tbar, int* drafter_out,
                                     int* T_out, double* latency_out) {
    if (n_models < 1 || !cost || !alpha || Tbar < 1 || !drafter_out || !T_out || !latency_out) {
        hsd_set_error("hsd_best_single_draft: bad arguments");
        return HSD_EINVAL;
    }
    const int K = n_models - 1;
    double best = cost[K];
    int bi = -1, bt = 0;
    for (int i = 0; i < K; ++i) {
        if (!valid_rate(alpha[i * n_models + K]) || !(cost[i] > 0.0)) { hsd_set_error("hsd_best_single_draft: bad cost / rate for model %d", i); return HSD_EINVAL; }
        for (int T = 1; T <= Tbar; ++T) {
            const double v = top_factor(alpha[i * n_models + K], T) * (cost[K] + T * cost[i]);
            if (v < best) { best = v; bi = i; bt = T; }
        }
    }
    *drafter_out = bi;
    *T_out = bt;
    *latency_out = best;
    return HSD_OK;
}
