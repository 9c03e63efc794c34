"""Expected latency of a hierarchy and the choice of the best one (Sec. 3.3, Sec. 4).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Notation follows the paper: models M_0..M_K with costs c_i, acceptance rates
alpha_{i,j} (i < j), parameters T_0..T_{K-1}; acceptances are IID (Sec. 2).

 * gamma(alpha, T_i, T_j): expected number of draft+verify rounds a level needs
   to collect T_j tokens when it is fed T_i draft tokens per round (definition in
   Sec. 3.3).  A round yields n+1 tokens, n = number of accepted drafts, a
   geometric variable truncated at T_i.  The paper estimates gamma empirically;
   here it is the exact value of that definition (a small recursion over the
   number of tokens still missing).
 * latency_literal: Thm 3.2 / Cor. 4.1 exactly as printed, in the nested form of
   the path-cost expansion in the proof of Thm 4.3.
 * latency_exact: expectation of Alg. 1 as written, where a level returns all the
   tokens it collected (at least T_idx), so the level above receives batches of
   varying length.  Thm 3.2 plugs in exactly T_idx and therefore differs
   slightly for K >= 2.
 * select_hierarchy: min over (sigma, T) of the literal latency with T <= Tbar,
   the HSD problem of Sec. 4.2.  The reduction graph of Sec. 4.3 is acyclic apart
   from its zero-cost self-loops, so the cheapest augmented path is found by
   dynamic programming over the vertices (M_i, j) from the smallest model up;
   edge multipliers and costs are those of the paper's edge table.
 * monte_carlo: Alg. 1 with each acceptance replaced by a biased coin and each
   pass by a fixed cost (the device the paper's App. B.2 ablation uses).

Parity unpinned: rows 3-6 of the paper's two worked tables (App. B.3); the
paper's gamma there was an empirical estimate that the text does not give.
"""
import itertools
from functools import lru_cache


def top_factor(alpha, T):
    """(1 - alpha) / (1 - alpha^(T+1)): reciprocal of the expected tokens per target round."""
    if alpha >= 1.0:
        return 1.0 / (T + 1)
    return (1.0 - alpha) / (1.0 - alpha ** (T + 1))


def accepted_pmf(alpha, t):
    """P(n accepted out of t drafted), n = 0..t: alpha^n (1-alpha) for n < t, alpha^t for n = t."""
    return [alpha ** n * (1.0 - alpha) for n in range(t)] + [alpha ** t]


@lru_cache(maxsize=None)
def gamma(alpha, Ti, Tj):
    pmf = accepted_pmf(alpha, Ti)
    E = [0.0] * (Tj + Ti + 2)                      # E[c] = 0 for c >= Tj
    for c in range(Tj - 1, -1, -1):
        E[c] = 1.0 + sum(pmf[n] * E[c + n + 1] for n in range(Ti + 1))
    return E[0]


def latency_literal(costs, alphas, T):
    """costs c_0..c_K, alphas[i] = alpha_{i,i+1} (K values), T_0..T_{K-1}."""
    K = len(costs) - 1
    if K == 0:
        return costs[0]
    inner = T[0] * costs[0]
    for n in range(1, K):
        inner = gamma(alphas[n - 1], T[n - 1], T[n]) * (costs[n] + inner)
    return top_factor(alphas[K - 1], T[K - 1]) * (costs[K] + inner)


def latency_exact(costs, alphas, T):
    """Expected cost per emitted token of Alg. 1 as written (batches may exceed T_idx)."""
    K = len(costs) - 1
    if K == 0:
        return costs[0]
    batch = {T[0]: 1.0}                            # distribution of the batch length a level returns
    cost = T[0] * costs[0]
    for idx in range(1, K):
        a, need = alphas[idx - 1], T[idx]
        gain = {}                                  # tokens gained per round: n + 1
        for b, pb in batch.items():
            for n, pn in enumerate(accepted_pmf(a, b)):
                gain[n + 1] = gain.get(n + 1, 0.0) + pb * pn
        rounds = {}
        final = {}
        for c in range(need - 1, -1, -1):
            r, f = 1.0, {}
            for g, pg in gain.items():
                if c + g >= need:
                    f[c + g] = f.get(c + g, 0.0) + pg
                else:
                    r += pg * rounds[c + g]
                    for k, pk in final[c + g].items():
                        f[k] = f.get(k, 0.0) + pg * pk
            rounds[c], final[c] = r, f
        cost = rounds[0] * (cost + costs[idx])     # Wald: rounds is a stopping time
        batch = final[0]
    a = alphas[K - 1]
    tokens = sum(pb * (1.0 / top_factor(a, b)) for b, pb in batch.items())
    return (cost + costs[K]) / tokens


def monte_carlo(costs, alphas, T, n_rounds, rng):
    """Simulated cost per token over n_rounds calls of HSD(K, .) with coin-flip acceptances."""
    K = len(costs) - 1

    def n_accepted(a, t):
        n = 0
        while n < t and rng.random() < a:
            n += 1
        return n

    def run(idx):                                  # returns (tokens, cost)
        if idx == 0:
            return T[0], T[0] * costs[0]
        if idx == K:
            b, c = run(idx - 1)
            return n_accepted(alphas[idx - 1], b) + 1, c + costs[idx]
        count, cost = 0, 0.0
        while count < T[idx]:
            b, c = run(idx - 1)
            count += n_accepted(alphas[idx - 1], b) + 1
            cost += c + costs[idx]
        return count, cost

    tok = cst = 0.0
    for _ in range(n_rounds):
        t, c = run(K)
        tok += t
        cst += c
    return cst / tok


def select_hierarchy(cost, alpha, Tbar, monotone=True):
    """cost[0..K], alpha[i][j] for i < j.  Returns (latency, sigma, T): sigma ascending model
    indices ending in K (just [K] when plain decoding is best).  monotone=True keeps the paper's
    edge set (M_i, j) -> (M_k, l) with l <= j."""
    K = len(cost) - 1
    g = {}                                          # g[(i, j)] = (cost of one batch from level (i, j), (k, l) below or None)
    for i in range(K):
        for j in range(1, Tbar + 1):
            best, arg = j * cost[i], None
            for k in range(i):
                for l in range(1, (j if monotone else Tbar) + 1):
                    v = gamma(alpha[k][i], l, j) * (cost[i] + g[(k, l)][0])
                    if v < best:
                        best, arg = v, (k, l)
            g[(i, j)] = (best, arg)
    best, arg = cost[K], None
    for i in range(K):
        for j in range(1, Tbar + 1):
            v = top_factor(alpha[i][K], j) * (cost[K] + g[(i, j)][0])
            if v < best:
                best, arg = v, (i, j)
    sigma, T = [K], []
    while arg is not None:
        sigma.append(arg[0])
        T.append(arg[1])
        arg = g[arg][1]
    return best, sigma[::-1], T[::-1]


def select_bruteforce(cost, alpha, Tbar, monotone=True):
    """Same optimum by enumerating every subset sigma ending in K and every T in [1, Tbar]^(|sigma|-1)."""
    K = len(cost) - 1
    best = (cost[K], [K], [])
    for r in range(1, K + 1):
        for sub in itertools.combinations(range(K), r):
            sig = list(sub) + [K]
            cs = [cost[i] for i in sig]
            al = [alpha[sig[i]][sig[i + 1]] for i in range(r)]
            for T in itertools.product(range(1, Tbar + 1), repeat=r):
                if monotone and any(T[i] > T[i + 1] for i in range(r - 1)):
                    continue
                v = latency_literal(cs, al, list(T))
                if v < best[0] - 1e-15:
                    best = (v, sig, list(T))
    return best


def best_single_draft(cost, alpha, Tbar):
    """The paper's single-draft baseline (Sec. 5.2): one drafter i and T minimising
    (c_K + T c_i) (1 - alpha) / (1 - alpha^(T+1))."""
    K = len(cost) - 1
    best = (cost[K], None, None)
    for i in range(K):
        for T in range(1, Tbar + 1):
            v = top_factor(alpha[i][K], T) * (cost[K] + T * cost[i])
            if v < best[0]:
                best = (v, i, T)
    return best
