"""Pins of the oracle's acceptance-rate calibration (Sec. 2 acceptance probability, Sec. 5.1 estimate)."""
import numpy as np

from oracle import calibrate, decoder, specsample
from paper_2510_19705_amd import inputs
from helpers import oracle_decoder


def _rows(n, V, seed):
    rng = np.random.default_rng(seed)
    z = rng.standard_normal((n, V)) * 2
    e = np.exp(z - z.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def test_overlap_is_the_acceptance_probability_of_alg2():
    """sum_x q(x) * P[u q(x) < p(x)] with u uniform on the 2^-24 grid of the oracle's accept test, evaluated exactly
    by counting grid points, equals sum min(p, q) up to the grid's resolution: ties the overlap to Alg. 2's rule."""
    V = 40
    p, q = _rows(2, V, 3).astype(np.float32)
    total = 0.0
    grid = 1 << 24
    for x in range(V):
        px, qx = float(p[x]), float(q[x])
        # number of u = k / 2^24 with fl32(u * q) < p: found by bisection on the oracle's own test (monotone in u)
        lo, hi = 0, grid                      # accept(lo) may be true, accept(hi) treated as false
        if not specsample.accept_test(0.0, px, qx):
            cnt = 0
        else:
            while hi - lo > 1:
                mid = (lo + hi) // 2
                if specsample.accept_test(mid / grid, px, qx):
                    lo = mid
                else:
                    hi = mid
            cnt = lo + 1
        total += float(q[x]) * cnt / grid
    assert abs(total - calibrate.overlap(p, q)) < 1e-6


def test_overlap_identities():
    V = 300
    r = _rows(4, V, 5)
    for i in range(4):
        assert abs(calibrate.overlap(r[i], r[i]) - 1) < 1e-12
        for j in range(4):
            assert abs(calibrate.overlap(r[i], r[j]) - (1 - calibrate.total_variation(r[i], r[j]))) < 1e-12
            assert calibrate.overlap(r[i], r[j]) == calibrate.overlap(r[j], r[i])
    onehot_a, onehot_b = np.zeros(V), np.zeros(V)
    onehot_a[3] = onehot_b[7] = 1
    assert calibrate.overlap(onehot_a, onehot_b) == 0 and calibrate.overlap(onehot_a, onehot_a) == 1
    # closed form on two-point distributions
    assert abs(calibrate.overlap([0.3, 0.7], [0.6, 0.4]) - 0.7) < 1e-15


def test_acceptance_matrix_of_decoder_exits():
    """Teacher-forced rows of every exit: matrix symmetric with unit diagonal, the triangle inequality of the
    appendix holds, deeper exits are closer to the target than shallow ones on the synthetic weights, and the rows
    equal what the HSD levels themselves compute for the same contexts (next_dists)."""
    shape = inputs.SHAPES["tiny"]
    w = inputs.make_weights(shape, seed=7, bf16=False)
    dec = oracle_decoder(shape, w, 64)
    toks = inputs.make_prompt(shape["vocab"], 40, seed=8)
    exits = (2, 4, 8)
    rows = calibrate.exit_distributions(dec, exits, toks, 16, 1.0)
    assert rows.shape == (3, 24, shape["vocab"]) and rows.dtype == np.float32
    alpha = calibrate.acceptance_matrix(rows)
    assert np.allclose(alpha, alpha.T) and np.allclose(np.diag(alpha), 1)
    assert calibrate.triangle_violation(alpha) <= 1e-9
    assert alpha[1, 2] > alpha[0, 2]                       # exit 4 agrees with the target more than exit 2
    assert 0 < alpha[0, 2] < 1
    lv = decoder.Level(dec, 4, 1.0)
    dec.reset()
    d = lv.next_dists([int(t) for t in toks[:30]], 3)       # rows for contexts of 28, 29, 30 tokens = positions 27..29
    assert np.array_equal(d, rows[1, 27 - 16:30 - 16])


def test_triangle_violation_detects_a_bad_matrix():
    a = np.array([[1, 0.9, 0.1], [0.9, 1, 0.9], [0.1, 0.9, 1]])     # 0.9 + 0.9 > 0.1 + 1
    assert calibrate.triangle_violation(a) > 0.6
