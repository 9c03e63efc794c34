"""Pins of the oracle's synthetic distilled drafters (noise generator and its effect on acceptance)."""
import math

import numpy as np

from oracle import calibrate, decoder, distill, hsd as ohsd, philox, specsample
from paper_2510_19705_amd import inputs
from helpers import oracle_decoder


def test_noise_is_standard_normal_and_addressed_by_level_and_position():
    n = distill.gaussian_noise(7, 1, 33, 200001)
    assert n.shape == (200001,)
    assert abs(n.mean()) < 4 / math.sqrt(len(n)) and abs(n.var() - 1) < 4 * math.sqrt(2 / len(n))
    assert abs((np.abs(n) < 1).mean() - 0.6827) < 0.005 and abs((np.abs(n) < 2).mean() - 0.9545) < 0.003
    # kurtosis of a normal is 3; a uniform or a wrongly scaled Box-Muller would miss it
    assert abs(((n - n.mean()) ** 4).mean() / n.var() ** 2 - 3) < 0.05
    assert np.array_equal(n[:777], distill.gaussian_noise(7, 1, 33, 777))           # a prefix does not depend on the length
    for other in (distill.gaussian_noise(8, 1, 33, 999), distill.gaussian_noise(7, 2, 33, 999), distill.gaussian_noise(7, 1, 34, 999)):
        assert abs(np.corrcoef(n[:999], other)[0, 1]) < 0.15
    # one value by hand from the block's words
    w = philox.philox4x32_10(np.array([5, 33, 1 | 0x80000000, distill.NOISE_TAG], dtype=np.uint64), (7, 0))
    u1, u2 = (float(w[2]) + 0.5) / 2 ** 32, (float(w[3]) + 0.5) / 2 ** 32
    assert abs(n[22] - math.sqrt(-2 * math.log(u1)) * math.cos(2 * math.pi * u2)) < 1e-12
    assert abs(n[23] - math.sqrt(-2 * math.log(u1)) * math.sin(2 * math.pi * u2)) < 1e-12


def test_distilled_levels_give_graded_acceptance_and_leave_the_target_law():
    """More noise, less overlap with the source; at temperature 0 the generated stream is the target's greedy stream
    whatever the drafters are (Thm 3.1 in its deterministic special case)."""
    shape = inputs.SHAPES["tiny"]
    w = inputs.make_weights(shape, seed=1, bf16=False)
    dec = oracle_decoder(shape, w, 128)
    small = dict(n_layers=2, d=128, n_q=2, n_kv=1, hd=64, ffn=384, vocab=shape["vocab"])
    dec_a = oracle_decoder(small, inputs.make_weights(small, seed=51, bf16=False), 128)
    prompt = [int(t) for t in inputs.make_prompt(shape["vocab"], 24, seed=10)]
    target = decoder.Level(dec, 8, 1.0)
    p = target.next_dists(prompt, 4)
    overlaps = []
    for std in (0.25, 0.5, 1.0, 2.0):
        lv = distill.DistilledLevel(dec_a, 2, target, 0, std, 3, 1.0)
        q = lv.next_dists(prompt, 4)
        overlaps.append(np.mean([calibrate.overlap(p[r], q[r]) for r in range(4)]))
    assert overlaps[0] > overlaps[1] > overlaps[2] > overlaps[3] and overlaps[0] > 0.85 and 0.3 < overlaps[2] < 0.85
    # same context, same rows, whatever the batch of rows asked for
    lv = distill.DistilledLevel(dec_a, 2, target, 0, 1.0, 3, 1.0)
    assert np.array_equal(lv.next_dists(prompt, 4)[3], lv.next_dists(prompt, 1)[0])
    # temperature 0
    t0 = decoder.Level(dec, 8, 0.0)
    levels = [distill.DistilledLevel(dec_a, 2, t0, 0, 1.0, 3, 0.0), distill.DistilledLevel(dec, 4, t0, 1, 0.5, 3, 0.0), t0]
    o = ohsd.HSD(levels, (3, 2), specsample.PhiloxChooser(1))
    got = o.generate(prompt, 24)
    dec.reset()
    greedy = ohsd.HSD([decoder.Level(dec, 8, 0.0)], (), specsample.PhiloxChooser(1)).generate(prompt, 24)
    assert got == greedy
    assert 0 < o.accepted[2] < o.drafted[2]


def test_a_chain_of_synthetic_levels_adds_one_noise_term_per_step():
    """A level whose source is synthetic too: its logits are the real network's plus the noise rows of every level of
    the chain (each identified by its own level index), so neighbours overlap more than the ends of the chain, and
    the overlap of the ends equals that of a single level with the summed noise."""
    shape = inputs.SHAPES["tiny"]
    w = inputs.make_weights(shape, seed=1, bf16=False)
    dec = oracle_decoder(shape, w, 128)
    prompt = [int(t) for t in inputs.make_prompt(shape["vocab"], 24, seed=10)]
    target = decoder.Level(dec, 8, 1.0)
    mid = distill.DistilledLevel(dec, 4, target, 1, 0.5, 3, 1.0)
    low = distill.DistilledLevel(dec, 2, mid, 0, 0.75, 3, 1.0)
    z_t = np.array(dec.next_logits(prompt, 3, 8), dtype=np.float64)
    z_low = low.logit_rows(prompt, 3)
    for r in range(3):
        pos = len(prompt) - 3 + r
        want = z_t[r] + 0.5 * distill.gaussian_noise(3, 1, pos, shape["vocab"]) + 0.75 * distill.gaussian_noise(3, 0, pos, shape["vocab"])
        assert np.allclose(z_low[r], want, rtol=0, atol=1e-12)
    p, pm, pl = target.next_dists(prompt, 3), mid.next_dists(prompt, 3), low.next_dists(prompt, 3)
    ov = lambda a, b: np.mean([calibrate.overlap(a[r], b[r]) for r in range(3)])
    assert ov(pl, pm) > ov(pl, p) and ov(pm, p) > ov(pl, p)
