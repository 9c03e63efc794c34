"""HSD recursion (Alg. 1) and the generation loop around it.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

What Alg. 1 computes, written as levels that gather tokens up to a quota: level 0
drafts T_0 tokens one at a time and keeps each full distribution; an
intermediate level idx repeatedly asks the level below for a batch, verifies it
(Alg. 2) and keeps the verified tokens until it holds at least T_idx of them,
then hands up ALL it holds (so the level above may see more than T_idx tokens:
Alg. 1 returns its whole list, not a prefix; the footnote to the definition of
gamma in Sec. 3.3 notes the same); the top level K does one such batch +
verification.  Every call starts with nothing gathered, so what a lower level
held beyond a rejection is discarded.  Pinned by exact enumeration of the output
law (Thm 3.1) in tests/test_oracle_hsd.py.

A level is anything with `next_dists(context, n_rows)` returning the fp32 rows
p(. | context[:len-n_rows+1+r]) for r = 0..n_rows-1.  Random decisions go
through a chooser (specsample.PhiloxChooser, or exact.ScriptedChooser for
exact enumeration): `call` counts a level's Verify calls, or draft steps at
level 0.

`truncate=True` is the variant the latency formula of Thm 3.2 describes literally: an intermediate level hands up
exactly T_idx tokens (what it collected beyond that is dropped), so every Verify sees exactly T drafts.  The
counter `tested` (accept tests evaluated: up to and including the first rejection) gives the per-test acceptance
frequency accepted / tested that the IID ablation of the appendix plugs into its coin.
"""
from . import specsample


class HSD:
    def __init__(self, levels, T, chooser, truncate=False):
        assert len(T) == len(levels) - 1 and all(t >= 1 for t in T)
        self.truncate = truncate
        self.levels = levels
        self.K = len(levels) - 1
        self.T = list(T)
        self.chooser = chooser
        self.calls = [0] * len(levels)
        # counters, for acceptance-rate and pass-count comparisons with the library
        self.passes = [0] * len(levels)
        self.drafted = [0] * len(levels)       # draft tokens offered to level idx's Verify
        self.accepted = [0] * len(levels)      # of those, accepted
        self.pass_rows = [0] * len(levels)
        self.tested = [0] * len(levels)        # accept tests evaluated at level idx

    def _verify(self, idx, draft_tokens, draft_probs, context):
        t = len(draft_tokens)
        p_rows = self.levels[idx].next_dists(list(context) + list(draft_tokens), t + 1)
        self.passes[idx] += 1
        call = self.calls[idx]
        self.calls[idx] += 1
        n, m = specsample.verify(p_rows, draft_probs, draft_tokens, self.chooser, idx, call)
        self.drafted[idx] += t
        self.accepted[idx] += n
        self.tested[idx] += n + (1 if n < t else 0)
        return list(draft_tokens[:n]) + [m], [p_rows[i] for i in range(n + 1)]

    def _draft(self, context, how_many):
        """Level 0 of Alg. 1: `how_many` tokens one after the other, each with the full row it was drawn from."""
        drawn, rows = [], []
        for _ in range(how_many):
            row = self.levels[0].next_dists(list(context) + drawn, 1)[0]
            self.passes[0] += 1
            step = self.calls[0]
            self.calls[0] += 1
            drawn.append(self.chooser.sample(0, step, 0, row, None))
            rows.append(row)
        return drawn, rows

    def run(self, idx, context):
        """HSD(idx, context) -> (tokens, probs).

        Written as "a level gathers verified tokens until it has its quota": the lowest level's quota is T_0 drafts;
        an intermediate level keeps asking the level below for a batch behind what it has gathered so far and keeps
        what its own Verify lets through, until it holds T_idx tokens, and hands up everything it holds (or exactly
        T_idx with truncate); the target's quota is one batch."""
        if idx == 0:
            return self._draft(context, self.T[0] if self.K > 0 else 1)
        top = idx == self.K
        gathered, rows = [], []
        while top or len(gathered) < self.T[idx]:
            behind = list(context) + gathered
            batch, batch_rows = self.run(idx - 1, behind)
            kept, kept_rows = self._verify(idx, batch, batch_rows, behind)
            gathered += kept
            rows += kept_rows
            if top:
                break
        if self.truncate and not top:
            gathered, rows = gathered[:self.T[idx]], rows[:self.T[idx]]
        return gathered, rows

    def generate(self, prompt, n_tokens):
        """Call HSD(K, context) until n_tokens are produced; the last round is cut at n_tokens.
        With a single level (K = 0) this is plain autoregressive sampling from that model."""
        out = []
        while len(out) < n_tokens:
            toks, _ = self.run(self.K, list(prompt) + out)
            out.extend(toks)
        return out[:n_tokens]
