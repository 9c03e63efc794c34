"""Speculative-sampling rule and Verify (Sec. 2; Alg. 2, App. B.1).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper fixes the rule (accept x ~ q with probability min(1, p(x)/q(x));
on rejection resample from max(0, p-q) normalised) but not its arithmetic.
Readings taken here, each implemented independently by the HIP library:

 * accept test: u on a 2^-24 grid in [0,1); accept iff fl32(u * q(x)) < p(x).
   One fp32 multiply and one compare, no division.  p(x)=0 never accepts,
   q(x)=0<p(x) always accepts.  Differs from Alg. 2's "r > p/q rejects"
   only on a null set.
 * sampling from a non-negative weight row r (r = p for the bonus token and
   for drafting, r = max(0, p-q) in fp32 after a rejection): integer weights
   w_x = floor(r_x * 2^62) (exact: r_x is an fp32 in [0,1]), S = sum w_x,
   threshold = floor(S * U / 2^32) with U a 32-bit word, token = smallest x
   whose inclusive prefix sum exceeds the threshold.  Integer sums are
   associative, so any reduction order gives the same token.
   If the residual row sums to zero (p == q to rounding, reachable only after
   a numerically marginal rejection) the row p is used instead.
"""
import numpy as np

from . import philox

_TWO62 = float(2 ** 62)


def accept_test(u, p_x, q_x):
    """Sec. 2 rule with the fp32 reading above."""
    return bool(np.float32(np.float32(u) * np.float32(q_x)) < np.float32(p_x))


def residual_row(p, q):
    """max(0, p - q) element-wise in fp32 (numerator of p' in Sec. 2)."""
    p = np.asarray(p, dtype=np.float32)
    q = np.asarray(q, dtype=np.float32)
    return np.maximum(np.float32(0), (p - q).astype(np.float32))


def fixed_weights(r):
    """w_x = floor(r_x * 2^62) as unsigned 64-bit integers."""
    r = np.asarray(r, dtype=np.float32).astype(np.float64)
    return np.floor(r * _TWO62).astype(np.uint64)


def sample_weights(w, U32, margins=None):
    """Token index from integer weights and one 32-bit word; None if all weights are zero.
    `margins` (a list) receives the distance of the threshold to the nearer end of the chosen
    token's interval, as a fraction of the total: how far a perturbed row could move it."""
    S = int(np.sum(w, dtype=np.uint64))
    if S == 0:
        return None
    thr = (S * int(U32)) >> 32
    pref = np.cumsum(w, dtype=np.uint64)
    m = int(np.searchsorted(pref, np.uint64(thr), side="right"))
    if margins is not None:
        lo = int(pref[m - 1]) if m > 0 else 0
        margins.append(min(thr - lo, int(pref[m]) - thr) / S)
    return m


def sample_row(p, q, U32, margins=None):
    """m ~ Normalize(max(0, p - q)) (q given) or m ~ p (q None), fixed-point rule."""
    if q is not None:
        m = sample_weights(fixed_weights(residual_row(p, q)), U32, margins)
        if m is not None:
            return m
    m = sample_weights(fixed_weights(np.asarray(p, dtype=np.float32)), U32, margins)
    if m is None:
        raise ValueError("distribution row is identically zero")
    return m


class PhiloxChooser:
    """Random decisions of Alg. 1/2 drawn from Philox blocks (see philox.py)."""

    def __init__(self, seed):
        self.seed = int(seed)
        self.accept_margins = []      # |u q(x) - p(x)| / max(u q(x), p(x)) of every accept test
        self.sample_margins = []      # see sample_weights

    def accept(self, level, call, i, p_x, q_x):
        w = philox.draw(self.seed, level, call, i)
        u = philox.uniform24(w[0])
        lhs, rhs = float(np.float32(u) * np.float32(q_x)), float(p_x)
        self.accept_margins.append(abs(lhs - rhs) / max(lhs, rhs, 1e-30))
        return accept_test(u, p_x, q_x)

    def sample(self, level, call, slot, p, q):
        w = philox.draw(self.seed, level, call, slot)
        return sample_row(p, q, int(w[1]), self.sample_margins)


class IIDChooser(PhiloxChooser):
    """The ablation of the appendix "Examining the assumptions of HSD": Alg. 2's test on each draft is replaced by a
    biased coin, P[accept] = alpha[level] whatever p and q are (the coin uses the same Philox word as the real test
    would; the corrected / bonus token is drawn as before).  alpha is indexed by the verifying level."""

    def __init__(self, seed, alpha):
        super().__init__(seed)
        self.alpha = [np.float32(a) for a in alpha]

    def accept(self, level, call, i, p_x, q_x):
        w = philox.draw(self.seed, level, call, i)
        return bool(np.float32(philox.uniform24(w[0])) < self.alpha[level])


def verify(p_rows, q_rows, x, chooser, level, call):
    """Alg. 2 after the verifier pass: p_rows = (p_1..p_{t+1}), q_rows = (q_1..q_t),
    x = (x_1..x_t).  Returns (n, m): number of accepted draft tokens and the
    corrected / bonus token.  Output tokens are x_1..x_n, m and output probs are
    p_1..p_{n+1} (rows of p_rows), as Alg. 2 returns them."""
    t = len(x)
    assert len(p_rows) == t + 1 and len(q_rows) == t
    n = t
    for i in range(t):
        xi = int(x[i])
        if not chooser.accept(level, call, i, p_rows[i][xi], q_rows[i][xi]):
            n = i
            break
    if n < t:
        m = chooser.sample(level, call, t, p_rows[n], q_rows[n])
    else:
        m = chooser.sample(level, call, t, p_rows[t], None)
    return n, m
