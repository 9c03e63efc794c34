"""Empirical acceptance rates between candidate models, as the selection of Sec. 4 needs them.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Sec. 2: a draft x ~ q is accepted by a verifier with distribution p with probability
    alpha_c = sum_x q(x) min(1, p(x) / q(x)) = sum_x min(p(x), q(x)) = 1 - TV(p, q),
TV = half the L1 distance.  Sec. 5.1 estimates alpha_{i,j} = E_c[alpha_c] by running the network
over sample contexts, keeping every candidate exit's output distribution at every position and
averaging that expression over the positions; the hierarchy-example appendix notes the triangle
inequality alpha_{i,j} + alpha_{j,k} <= alpha_{i,k} + 1 the estimates inherit from TV.

Everything here is the definition written out in fp64.  A position's row for exit e is the
distribution of the next token given the tokens up to and including that position.
"""
import numpy as np

from . import decoder as _decoder


def overlap(p, q):
    """sum_x min(p(x), q(x)) of two distribution rows (Sec. 2, acceptance rate of one context)."""
    return float(np.minimum(np.asarray(p, dtype=np.float64), np.asarray(q, dtype=np.float64)).sum())


def total_variation(p, q):
    """Half the L1 distance; overlap = 1 - TV for rows that each sum to one."""
    return 0.5 * float(np.abs(np.asarray(p, dtype=np.float64) - np.asarray(q, dtype=np.float64)).sum())


def exit_distributions(dec, exits, tokens, n_ctx, temperature):
    """Rows [len(exits), len(tokens) - n_ctx, V] (fp32, as the library stores them): exit e's distribution of
    the next token after each of the positions n_ctx .. len(tokens) - 1, teacher-forced on `tokens`."""
    toks = [int(t) for t in tokens]
    out = []
    for e in exits:
        dec.reset()
        z = dec.forward(toks, 0, e)[n_ctx:]
        out.append(_decoder.distributions(z, temperature))
    return np.stack(out)


def acceptance_matrix(rows):
    """alpha[i, j] = mean over positions of overlap(rows[i, pos], rows[j, pos]); symmetric, ones on the diagonal
    (up to the rows' own rounding)."""
    n = rows.shape[0]
    alpha = np.ones((n, n))
    for i in range(n):
        for j in range(i + 1, n):
            a = np.mean([overlap(rows[i, t], rows[j, t]) for t in range(rows.shape[1])])
            alpha[i, j] = alpha[j, i] = a
    return alpha


def triangle_violation(alpha):
    """Largest alpha[i,j] + alpha[j,k] - alpha[i,k] - 1 over distinct triples (<= 0 for exact rows)."""
    n = alpha.shape[0]
    worst = -np.inf
    for i in range(n):
        for j in range(n):
            for k in range(n):
                if len({i, j, k}) == 3:
                    worst = max(worst, alpha[i, j] + alpha[j, k] - alpha[i, k] - 1.0)
    return worst
