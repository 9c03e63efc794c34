"""Pins for oracle/hsd.py (CPU only): Thm 3.1 by exact enumeration, temperature-0 equivalence
with greedy decoding of the target, and the batch structure of Alg. 1."""
import numpy as np
import pytest

from oracle import decoder, exact, hsd, specsample
from paper_2510_19705_amd import inputs


@pytest.mark.parametrize("K,V,T,N,order", [
    (1, 3, (1,), 2, 1),
    (1, 3, (2,), 2, 2),
    (1, 2, (3,), 3, 1),
    (2, 2, (1, 1), 2, 1),
    (2, 2, (2, 1), 2, 1),      # T_1 < T_0 is legal in Alg. 1
    (2, 2, (1, 2), 2, 2),
    (2, 3, (1, 2), 1, 1),
    (3, 2, (1, 1, 1), 1, 1),
])
def test_output_law_equals_target_law(K, V, T, N, order):
    """Thm 3.1: for any models and any T, the emitted tokens follow the target's distribution."""
    rng = np.random.default_rng(100 * K + 10 * V + sum(T))
    levels = [exact.TableLevel(V, order, rng) for _ in range(K + 1)]
    prompt = [1, 0]

    def run(ch):
        return tuple(hsd.HSD(levels, T, ch).generate(prompt, N))

    law, leaves = exact.explore(run)
    ref = exact.target_law(levels[K], prompt, N)
    assert abs(sum(law.values()) - 1.0) < 1e-10
    for y, pr in ref.items():
        assert abs(law.get(y, 0.0) - pr) < 1e-12, (y, leaves)


def test_planted_mistake_is_caught_by_the_enumeration():
    """The enumeration has teeth: sampling the corrected token from p instead of the residual
    breaks the law (so Thm 3.1 really pins that step)."""
    rng = np.random.default_rng(7)
    levels = [exact.TableLevel(3, 1, rng) for _ in range(2)]

    class Wrong(exact.ScriptedChooser):
        def sample(self, level, call, slot, p, q):
            return super().sample(level, call, slot, p, None)

    def run_with(cls):
        law, stack = {}, [()]
        while stack:
            script = stack.pop()
            ch = cls(script)
            out = tuple(hsd.HSD(levels, (2,), ch).generate([0], 1))
            law[out] = law.get(out, 0.0) + ch.prob
            taken = tuple(k for k, _ in ch.trace)
            for depth in range(len(script), len(ch.trace)):
                k, probs = ch.trace[depth]
                stack.extend(taken[:depth] + (alt,) for alt, pr in enumerate(probs) if alt != k and pr > 0)
        return law

    ref = exact.target_law(levels[1], [0], 1)
    good, bad = run_with(exact.ScriptedChooser), run_with(Wrong)
    assert max(abs(good[y] - ref[y]) for y in ref) < 1e-12
    assert max(abs(bad[y] - ref[y]) for y in ref) > 1e-3


SHAPE = dict(n_layers=4, d=32, n_q=4, n_kv=2, hd=8, ffn=64, vocab=50)


def _levels(temperature, exits, seed=1):
    w = inputs.make_weights(SHAPE, seed=seed, bf16=False)
    spec = decoder.Spec(SHAPE["n_layers"], SHAPE["d"], SHAPE["n_q"], SHAPE["n_kv"], SHAPE["hd"], SHAPE["ffn"],
                        SHAPE["vocab"], inputs.ROPE_BASE, inputs.EPS)
    dec = decoder.Decoder(spec, w, max_len=128)
    return [decoder.Level(dec, e, temperature) for e in exits]


@pytest.mark.parametrize("T", [(4, 2), (2, 4), (1, 1), (3, 3)])
def test_temperature_zero_stream_equals_greedy_target(T):
    """With one-hot rows every level accepts exactly the tokens that equal its own argmax and the
    corrected token is the verifier's argmax, so HSD must reproduce plain greedy decoding."""
    prompt = [int(v) for v in inputs.make_prompt(SHAPE["vocab"], 9, seed=3)]
    out = hsd.HSD(_levels(0, (1, 2, 4)), T, specsample.PhiloxChooser(5)).generate(prompt, 24)
    greedy = hsd.HSD(_levels(0, (4,)), (), specsample.PhiloxChooser(77)).generate(prompt, 24)
    assert out == greedy
    # and greedy is the textbook loop
    lv = _levels(0, (4,))[0]
    ctx = list(prompt)
    for _ in range(24):
        ctx.append(int(np.argmax(lv.decoder.next_logits(ctx, 1, 4)[0].astype(np.float32))))
    assert ctx[len(prompt):] == greedy


def test_batch_structure_of_alg1():
    """Level 0 returns exactly T_0 tokens; an intermediate level returns at least T_idx and stops at the
    first round that reaches it; probabilities come back one row per token."""
    levels = _levels(1.0, (1, 2, 4))
    h = hsd.HSD(levels, (3, 5), specsample.PhiloxChooser(11))
    prompt = [1, 2, 3, 4]
    t0, p0 = h.run(0, prompt)
    assert len(t0) == 3 and len(p0) == 3
    for _ in range(5):
        t1, p1 = h.run(1, prompt)
        assert 5 <= len(t1) <= 5 - 1 + 3 + 1 and len(p1) == len(t1)
        assert all(abs(float(r.sum()) - 1) < 1e-5 for r in p1)
    before = list(h.passes)
    tk, _ = h.run(2, prompt)
    assert h.passes[2] == before[2] + 1 and 1 <= len(tk)


def test_counters_track_acceptance():
    levels = _levels(1.0, (2, 4))
    h = hsd.HSD(levels, (4,), specsample.PhiloxChooser(3))
    out = h.generate([5, 6, 7], 40)
    assert len(out) == 40
    assert h.drafted[1] == 4 * h.passes[1] and 0 <= h.accepted[1] <= h.drafted[1]
    assert h.accepted[1] + h.passes[1] >= 40          # every target pass emits accepted + 1 tokens
