"""Exact enumeration of the output law of Alg. 1/2 on toy models (pin for Thm 3.1).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Thm 3.1 states that, for any models and any parameters T, the tokens HSD emits
follow the target model's distribution.  To check the oracle's Alg. 1/Alg. 2
code against that statement, the same code (hsd.HSD, specsample.verify) is run
with every random decision replaced by a scripted one, and all scripts are
explored depth-first, multiplying the exact probabilities of the decisions:
  accept x_i       with probability min(1, p_i(x_i)/q_i(x_i))      (Sec. 2)
  corrected token  ~ max(0, p-q) / sum max(0, p-q)                 (Sec. 2)
  bonus / draft    ~ p
The resulting law of the first N emitted tokens must equal prod_j p_K(y_j | prefix).
"""
import itertools

import numpy as np


class ScriptedChooser:
    """Replays `script` (a tuple of outcome indices), then takes the first outcome with
    non-zero probability; records every decision's outcome probabilities in `trace`."""

    def __init__(self, script):
        self.script = tuple(script)
        self.trace = []
        self.prob = 1.0

    def _choose(self, probs):
        k = self.script[len(self.trace)] if len(self.trace) < len(self.script) else \
            next(i for i, pr in enumerate(probs) if pr > 0)
        self.trace.append((k, probs))
        self.prob *= probs[k]
        return k

    def accept(self, level, call, i, p_x, q_x):
        a = 1.0 if q_x <= p_x else float(p_x) / float(q_x)
        return self._choose((a, 1.0 - a)) == 0

    def sample(self, level, call, slot, p, q):
        r = np.asarray(p, dtype=np.float64)
        if q is not None:
            r = np.maximum(0.0, r - np.asarray(q, dtype=np.float64))
        return self._choose(tuple(float(v) for v in r / r.sum()))


def explore(run):
    """run(chooser) -> hashable outcome.  Returns {outcome: probability} over all decision paths."""
    law = {}
    stack = [()]
    n_leaves = 0
    while stack:
        script = stack.pop()
        ch = ScriptedChooser(script)
        out = run(ch)
        n_leaves += 1
        law[out] = law.get(out, 0.0) + ch.prob
        taken = tuple(k for k, _ in ch.trace)
        for depth in range(len(script), len(ch.trace)):
            k, probs = ch.trace[depth]
            for alt, pr in enumerate(probs):
                if alt != k and pr > 0:
                    stack.append(taken[:depth] + (alt,))
    return law, n_leaves


class TableLevel:
    """Toy language model: the next-token distribution depends on the last `order` tokens only."""

    def __init__(self, vocab, order, rng, sharp=1.0):
        self.vocab, self.order = vocab, order
        self.table = {}
        for n in range(order + 1):
            for suf in itertools.product(range(vocab), repeat=n):
                self.table[suf] = rng.dirichlet(np.full(vocab, sharp))

    def dist(self, context):
        ctx = tuple(int(t) for t in context)
        return self.table[ctx[len(ctx) - min(self.order, len(ctx)):]]

    def next_dists(self, context, n_rows):
        L = len(context)
        return [self.dist(context[:L - n_rows + 1 + r]) for r in range(n_rows)]


def target_law(level, prompt, n_tokens):
    """prod_j p(y_j | prompt + y_<j) for every y in V^n_tokens."""
    law = {}
    for y in itertools.product(range(level.vocab), repeat=n_tokens):
        pr = 1.0
        for j in range(n_tokens):
            pr *= level.dist(list(prompt) + list(y[:j]))[y[j]]
        law[y] = pr
    return law
