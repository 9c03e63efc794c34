"""Pins for oracle/philox.py and oracle/specsample.py (CPU only)."""
import os

import numpy as np
import pytest

from oracle import exact, philox, specsample


def test_philox_known_answers(golden_dir):
    n = 0
    for line in open(os.path.join(golden_dir, "philox_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(v, 16) for v in line.split()]
        out = philox.philox4x32_10(w[0:4], w[4:6])
        assert [int(v) for v in out] == w[6:10]
        n += 1
    assert n == 3


def test_philox_vectorised_equals_scalar():
    ctr = np.array([[i, 7, 2, 0] for i in range(50)], dtype=np.uint64)
    many = philox.philox4x32_10(ctr, (123, 456))
    for i in range(50):
        assert (many[i] == philox.philox4x32_10(ctr[i], (123, 456))).all()
    assert (philox.draw((456 << 32) | 123, 2, 7, 5) == many[5]).all()


def test_uniform24_grid():
    assert philox.uniform24(0) == 0.0
    assert philox.uniform24(0xFFFFFFFF) == np.float32(1.0 - 2.0 ** -24)
    assert philox.uniform24(0x80000000) == 0.5


def _rows(V, seed, sharp=1.0):
    rng = np.random.default_rng(seed)
    p = rng.dirichlet(np.full(V, sharp)).astype(np.float32)
    q = rng.dirichlet(np.full(V, sharp)).astype(np.float32)
    return p, q


def test_accept_boundaries():
    assert not specsample.accept_test(0.0, 0.0, 0.5)          # p = 0 never accepts
    assert not specsample.accept_test(0.0, 0.0, 0.0)
    assert specsample.accept_test(0.999, 0.1, 0.0)            # q = 0 < p always accepts
    assert specsample.accept_test(np.float32(1 - 2.0 ** -24), 1.0, 1.0)   # one-hot rows, same token
    assert not specsample.accept_test(0.0, 0.0, 1.0)          # one-hot rows, different token
    assert specsample.accept_test(0.49, 0.25, 0.5) and not specsample.accept_test(0.5, 0.25, 0.5)


def test_accept_frequency_matches_sum_min():
    """Sec. 2: P(accept) = sum_x min(p, q) = 1 - sum |p - q| / 2."""
    V, N = 12, 20000
    p, q = _rows(V, 3)
    alpha = float(np.minimum(p.astype(np.float64), q.astype(np.float64)).sum())
    assert abs(alpha - (1 - 0.5 * np.abs(p.astype(np.float64) - q).sum())) < 1e-6
    rng = np.random.default_rng(0)
    xs = rng.choice(V, size=N, p=q.astype(np.float64) / q.astype(np.float64).sum())
    ch = specsample.PhiloxChooser(seed=99)
    acc = sum(ch.accept(1, c, 0, p[x], q[x]) for c, x in enumerate(xs))
    sigma = np.sqrt(alpha * (1 - alpha) / N)
    assert abs(acc / N - alpha) < 4 * sigma


def test_residual_normaliser_identity():
    """sum max(0, p - q) = 1 - sum min(p, q); the integer total tracks it to V * 2^-62 plus fp32 row error."""
    p, q = _rows(1000, 5)
    r = specsample.residual_row(p, q)
    p64, q64 = p.astype(np.float64), q.astype(np.float64)
    assert abs(r.astype(np.float64).sum() - (p64.sum() - np.minimum(p64, q64).sum())) < 1e-6
    S = int(specsample.fixed_weights(r).sum(dtype=np.uint64))
    assert abs(S * 2.0 ** -62 - r.astype(np.float64).sum()) <= 1000 * 2.0 ** -62 + 1e-15


def test_sample_weights_partition_of_the_word_range():
    """Direct definition on tiny integer weights: token x owns the sub-interval of thresholds
    [prefix_{x-1}, prefix_x); zero weights are never chosen."""
    w = np.array([1, 0, 2, 1], dtype=np.uint64) << np.uint64(60)
    got = [specsample.sample_weights(w, U) for U in (0, 2 ** 30 - 1, 2 ** 30, 3 * 2 ** 30 - 1, 3 * 2 ** 30, 2 ** 32 - 1)]
    assert got == [0, 0, 2, 2, 3, 3]
    assert specsample.sample_weights(np.zeros(4, dtype=np.uint64), 5) is None


def test_sample_row_law_chi2():
    """Empirical law of the corrected token -> p' of Sec. 2 (chi-square, V = 16)."""
    V, N = 16, 20000
    p, q = _rows(V, 11)
    r = np.maximum(0, p.astype(np.float64) - q)
    pprime = r / r.sum()
    ch = specsample.PhiloxChooser(seed=5)
    cnt = np.zeros(V)
    for c in range(N):
        cnt[ch.sample(2, c, 3, p, q)] += 1
    assert cnt[pprime == 0].sum() == 0
    sup = pprime > 0
    chi2 = ((cnt[sup] - N * pprime[sup]) ** 2 / (N * pprime[sup])).sum()
    assert chi2 < 45.0                      # 99.99 % quantile of chi2 with <= 15 dof is 44.3
    # bonus / draft sampling (q absent) follows p itself
    cnt = np.zeros(V)
    for c in range(N):
        cnt[ch.sample(0, c, 0, p, None)] += 1
    chi2 = ((cnt - N * p) ** 2 / (N * p)).sum()
    assert chi2 < 45.0


def test_sample_row_falls_back_to_p_when_residual_is_zero():
    p = np.array([0.25, 0.75], dtype=np.float32)
    assert specsample.sample_row(p, p.copy(), 0) == 0
    assert specsample.sample_row(p, p.copy(), 2 ** 32 - 1) == 1


def _verify_law(p_rows, q_rows, t):
    """Exact law of (n, output tokens) of Alg. 2 when x_i ~ q_i is drawn inside the enumeration."""
    def run(ch):
        x = [ch.sample(0, 0, i, q_rows[i], None) for i in range(t)]
        n, m = specsample.verify(p_rows, q_rows, x, ch, 1, 0)
        return (n, tuple(x[:n]) + (m,))
    return exact.explore(run)[0]


@pytest.mark.parametrize("t", [1, 2, 3])
def test_verify_expected_length_closed_form(t):
    """With context-independent p and q, E[#output tokens] = (1 - alpha^(t+1)) / (1 - alpha)
    (Leviathan et al., quoted in the proof of Thm 3.2)."""
    V = 3
    p, q = _rows(V, 21)
    p64, q64 = p.astype(np.float64), q.astype(np.float64)
    p64, q64 = p64 / p64.sum(), q64 / q64.sum()
    law = _verify_law([p64] * (t + 1), [q64] * t, t)
    assert abs(sum(law.values()) - 1) < 1e-12
    alpha = np.minimum(p64, q64).sum()
    e_len = sum(pr * (n + 1) for (n, _), pr in law.items())
    assert abs(e_len - (1 - alpha ** (t + 1)) / (1 - alpha)) < 1e-12


def test_verify_first_token_law_is_p1_and_rows_are_indexed_by_position():
    """Law of the first output token is p_1; of the second given the first is p_2 (rows differ per
    position, so an off-by-one in the residual row or the bonus row fails here)."""
    V, t = 3, 2
    rng = np.random.default_rng(8)
    p_rows = [rng.dirichlet(np.ones(V)) for _ in range(t + 1)]
    q_rows = [rng.dirichlet(np.ones(V)) for _ in range(t)]
    law = _verify_law(p_rows, q_rows, t)
    first = np.zeros(V)
    for (n, toks), pr in law.items():
        first[toks[0]] += pr
    assert np.allclose(first, p_rows[0], atol=1e-12)
    # P(at least 2 tokens and second = y) = P(first accepted) * p_2(y) summed over first tokens
    second = np.zeros(V)
    for (n, toks), pr in law.items():
        if len(toks) >= 2:
            second[toks[1]] += pr
    a1 = np.minimum(p_rows[0], q_rows[0]).sum()
    assert np.allclose(second, a1 * p_rows[1], atol=1e-12)
    third = np.zeros(V)
    for (n, toks), pr in law.items():
        if len(toks) == 3:
            third[toks[2]] += pr
    a2 = np.minimum(p_rows[1], q_rows[1]).sum()
    assert np.allclose(third, a1 * a2 * p_rows[2], atol=1e-12)
