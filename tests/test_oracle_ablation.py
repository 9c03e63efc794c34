"""Pins of the oracle's ablation modes (appendix "Examining the assumptions of HSD"; Thm 3.2): coin-flip acceptances
and the exactly-T variant of Alg. 1 against the closed-form latencies, neither of which shares code with them."""
import numpy as np
import pytest

from oracle import exact, hsd as ohsd, latency, philox, specsample


def _cost_per_token(o, costs, n_tokens):
    return sum(p * c for p, c in zip(o.passes, costs)) / n_tokens


def _levels(n, seed):
    rng = np.random.default_rng(seed)
    return [exact.TableLevel(6, 1, rng) for _ in range(n)]


def test_coin_frequency_is_alpha():
    """The coin accepts iff u < alpha with u on the 2^-24 grid: over all Philox draws of a run the frequency matches
    alpha, and the test ignores p and q."""
    ch = specsample.IIDChooser(5, [0.0, 0.37, 0.9])
    for level, a in ((1, 0.37), (2, 0.9)):
        hits = sum(ch.accept(level, call, i, 0.0, 1.0) for call in range(400) for i in range(10))
        assert abs(hits / 4000 - a) < 4 * np.sqrt(a * (1 - a) / 4000)
    u = philox.uniform24(philox.draw(5, 1, 0, 0)[0])
    assert ch.accept(1, 0, 0, 1.0, 0.0) == (np.float32(u) < np.float32(0.37))


@pytest.mark.parametrize("T,alphas,costs", [((3,), (0.7,), (1.0, 10.0)), ((4, 2), (0.8, 0.6), (1.0, 3.0, 20.0)),
                                            ((2, 3, 2), (0.9, 0.7, 0.5), (1.0, 2.0, 6.0, 30.0))])
def test_iid_runs_match_the_closed_forms(T, alphas, costs):
    """Alg. 1 driven by coins: cost per token = the exact expectation with overshoot (Alg. 1 as written), and, in the
    exactly-T variant, the printed formula of Thm 3.2.  20000 tokens; tolerance 2 %, several times the Monte-Carlo
    error."""
    n = 20000
    K = len(T)
    coin = [0.0] + list(alphas)
    for truncate, want in ((False, latency.latency_exact(costs, alphas, T)), (True, latency.latency_literal(costs, alphas, T))):
        o = ohsd.HSD(_levels(K + 1, 3), T, specsample.IIDChooser(11, coin), truncate=truncate)
        out = []
        while len(out) < n:
            toks, _ = o.run(K, [0] + out[-1:])
            out.extend(toks)
        got = _cost_per_token(o, costs, len(out))
        assert abs(got - want) < 0.02 * want, (truncate, got, want)
        # per-test acceptance frequency of every level is its coin
        for lvl in range(1, K + 1):
            assert abs(o.accepted[lvl] / o.tested[lvl] - alphas[lvl - 1]) < 0.02


def test_truncate_hands_up_exactly_T():
    rng = np.random.default_rng(1)
    lv = [exact.TableLevel(5, 1, rng) for _ in range(3)]
    o = ohsd.HSD(lv, (3, 2), specsample.PhiloxChooser(9), truncate=True)
    seen = []
    orig = o._verify

    def spy(idx, dt, dp, ctx):
        seen.append((idx, len(dt)))
        return orig(idx, dt, dp, ctx)
    o._verify = spy
    for _ in range(50):
        o.run(2, [0])
    assert {t for i, t in seen if i == 2} == {2} and {t for i, t in seen if i == 1} == {3}
    # without truncation the top level sometimes sees more than T_1 drafts
    o2 = ohsd.HSD(lv, (3, 2), specsample.PhiloxChooser(9))
    seen.clear()
    orig2 = o2._verify
    o2._verify = lambda idx, dt, dp, ctx: (seen.append((idx, len(dt))), orig2(idx, dt, dp, ctx))[1]
    for _ in range(50):
        o2.run(2, [0])
    assert max(t for i, t in seen if i == 2) > 2
