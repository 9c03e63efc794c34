"""Pins for oracle/latency.py (CPU only): closed forms, the paper's printed worked examples,
Monte-Carlo of Alg. 1 with coin-flip acceptances, brute force over hierarchies."""
import math
import os

import numpy as np
import pytest

from oracle import latency


def _load_examples(golden_dir):
    rows, cost, alpha = [], {}, {}
    for line in open(os.path.join(golden_dir, "latency_examples.txt")):
        w = line.split()
        if not w or w[0].startswith("#"):
            continue
        if w[0] == "cost":
            cost[w[1]] = [float(v) for v in w[2:]]
        elif w[0] == "alpha":
            alpha.setdefault(w[1], {})[int(w[2])] = w[3:]
        else:
            rows.append((w[0], int(w[1]), float(w[2]), float(w[3]), w[4]))
    mats = {}
    for name, r in alpha.items():
        a = [[0.0] * 6 for _ in range(6)]
        for i, vals in r.items():
            for jj, v in enumerate(vals):
                if v != "-":
                    a[i - 1][jj + 1] = float(v)
        mats[name] = a
    return rows, cost, mats


def test_gamma_closed_forms():
    for l in (1, 2, 5):
        assert latency.gamma(0.37, l, 1) == 1.0                       # one round always yields >= 1 token
        for j in (1, 3, 7):
            assert abs(latency.gamma(0.0, l, j) - j) < 1e-12          # nothing accepted: one token per round
            assert abs(latency.gamma(1.0, l, j) - math.ceil(j / (l + 1))) < 1e-12
    # T_i = 1, T_j = 2: first round gives 2 tokens w.p. alpha, else a second round is needed
    assert abs(latency.gamma(0.3, 1, 2) - (1 + 0.7)) < 1e-12


def test_gamma_monte_carlo():
    rng = np.random.default_rng(0)
    a, l, j, N = 0.7, 3, 8, 40000
    tot = 0
    for _ in range(N):
        c = r = 0
        while c < j:
            n = 0
            while n < l and rng.random() < a:
                n += 1
            c += n + 1
            r += 1
        tot += r
    assert abs(tot / N - latency.gamma(a, l, j)) < 0.02


def test_single_draft_closed_form():
    """K = 1 in Thm 3.2: (c_1 + T c_0)(1 - alpha)/(1 - alpha^(T+1)); literal == exact there."""
    for a, c0, c1, T in [(0.8, 4.0, 33.0, 5), (0.5, 256.0, 1024.0, 1), (0.0, 1.0, 2.0, 3), (1.0, 1.0, 7.0, 4)]:
        ref = (c1 + T * c0) / sum(a ** i for i in range(T + 1))
        assert abs(latency.latency_literal([c0, c1], [a], [T]) - ref) < 1e-12
        assert abs(latency.latency_exact([c0, c1], [a], [T]) - ref) < 1e-12


def test_printed_two_model_examples(golden_dir):
    """Sec. 3.4 / App. B.3, rows with 1 and 2 models: 33.00; 14.37 (T = 5, 2.2971x); 19.31 (T = 3, 1.7090x)."""
    rows, cost, mats = _load_examples(golden_dir)
    for name, n, lat, speed, pin in rows:
        c, a = cost[name][6 - n:], [r[6 - n:] for r in mats[name][6 - n:]]
        got, sigma, T = latency.select_hierarchy(c, a, 15)
        if pin == "exact":
            assert abs(got - lat) < 0.005 + 1e-9, (name, n, got)
            assert abs(c[-1] / got - speed) < 1e-4      # printed to four decimals (19.3089 -> 1.70905)
        else:   # context only: the paper's gamma was empirical; the optimum must still improve with n
            assert abs(got - lat) / lat < 0.12, (name, n, got)
    assert latency.select_hierarchy(cost["ex1"][4:], [r[4:] for r in mats["ex1"][4:]], 15)[2] == [5]
    assert latency.select_hierarchy(cost["ex2"][4:], [r[4:] for r in mats["ex2"][4:]], 15)[2] == [3]
    for name in ("ex1", "ex2"):
        seq = [latency.select_hierarchy(cost[name][6 - n:], [r[6 - n:] for r in mats[name][6 - n:]], 15)[0]
               for n in range(1, 7)]
        assert all(seq[i + 1] <= seq[i] + 1e-12 for i in range(5))


def test_exact_expectation_matches_monte_carlo_and_literal_overestimates():
    """For K >= 2 Alg. 1 hands up at least T_idx tokens; the exact expectation accounts for it and
    agrees with simulation, the printed formula (which plugs in exactly T_idx) is an upper bound here."""
    c, a, T = [0.25, 4.0, 33.0], [0.75, 0.8], [4, 8]
    ex = latency.latency_exact(c, a, T)
    lit = latency.latency_literal(c, a, T)
    mc = latency.monte_carlo(c, a, T, 60000, np.random.default_rng(1))
    assert abs(mc - ex) < 0.04
    assert lit > ex and (lit - ex) / ex < 0.06
    c, a, T = [1.0, 3.0, 9.0, 30.0], [0.6, 0.7, 0.8], [2, 3, 5]
    ex = latency.latency_exact(c, a, T)
    mc = latency.monte_carlo(c, a, T, 60000, np.random.default_rng(2))
    assert abs(mc - ex) / ex < 0.01


def test_literal_formula_is_the_sum_of_products_of_thm32():
    """Thm 3.2 as printed, sum_i c_i prod_{j>=i} R(alpha_{j-1,j}, j), equals the nested form."""
    c, a, T = [1.0, 3.0, 9.0, 30.0], [0.6, 0.7, 0.8], [2, 3, 5]
    K = 3

    def R(n):
        if n == K:
            return latency.top_factor(a[K - 1], T[K - 1])
        if n == 0:
            return T[0]
        return latency.gamma(a[n - 1], T[n - 1], T[n])

    s = sum(c[i] * math.prod(R(j) for j in range(i, K + 1)) for i in range(K + 1))
    assert abs(s - latency.latency_literal(c, a, T)) < 1e-12


@pytest.mark.parametrize("monotone", [True, False])
def test_selection_equals_brute_force(monotone):
    rng = np.random.default_rng(3)
    for trial in range(6):
        K = int(rng.integers(2, 5))
        cost = sorted(rng.uniform(0.05, 1.0, K).tolist()) + [float(rng.uniform(5, 30))]
        alpha = [[0.0] * (K + 1) for _ in range(K + 1)]
        for i in range(K + 1):
            for j in range(i + 1, K + 1):
                alpha[i][j] = float(rng.uniform(0.1, 0.95))
        Tbar = 3 if K == 4 else 4
        dp = latency.select_hierarchy(cost, alpha, Tbar, monotone)
        bf = latency.select_bruteforce(cost, alpha, Tbar, monotone)
        assert abs(dp[0] - bf[0]) < 1e-12
        cs = [cost[i] for i in dp[1]]
        al = [alpha[dp[1][i]][dp[1][i + 1]] for i in range(len(dp[1]) - 1)]
        assert abs(latency.latency_literal(cs, al, dp[2]) - dp[0]) < 1e-12     # path cost == L(sigma, T)


def test_abc_grid(golden_dir):
    """App. B.4 table: all 80 printed speed-ups within 0.01 (two-decimal print), hierarchy colours
    agree except at near-ties."""
    lines = [l.split() for l in open(os.path.join(golden_dir, "abc_grid.txt")) if l.strip() and not l.startswith("#")]
    costs_c = [float(v) for v in lines[0][1:]]
    table = {float(l[0]): [float(v) for v in l[1:]] for l in lines[1:] if l[0] != "hier"}
    hier = {float(l[1]): l[2:] for l in lines if l[0] == "hier"}
    assert len(table) == 10 and len(hier) == 10
    mism = 0
    for acb, row in table.items():
        for cc, printed, colour in zip(costs_c, row, hier[acb]):
            cost = [cc, 256.0, 1024.0]                                # C, B, A
            alpha = [[0, acb, max(0.0, acb + 0.5 - 1.0)], [0, 0, 0.5], [0, 0, 0]]
            lat, sigma, T = latency.select_hierarchy(cost, alpha, 15)
            assert abs(1024.0 / lat - printed) <= 0.0101, (acb, cc, 1024.0 / lat)
            name = {(1, 2): "AB", (0, 1, 2): "ABC", (0, 2): "AC"}[tuple(sigma)]
            mism += name != colour
    assert mism <= 2
    lat, sigma, T = latency.select_hierarchy([256.0, 1024.0], [[0, 0.5], [0, 0]], 15)
    assert T == [1] and abs(lat - 853.3333333) < 1e-6                 # A-B alone: speed-up 1.20


def test_best_single_draft():
    cost = [1.0, 4.0, 33.0]
    alpha = [[0, 0.7, 0.5], [0, 0, 0.8], [0, 0, 0]]
    lat, i, T = latency.best_single_draft(cost, alpha, 15)
    ref = min((latency.latency_literal([cost[k], 33.0], [alpha[k][2]], [t]), k, t) for k in (0, 1) for t in range(1, 16))
    assert (lat, i, T) == ref
