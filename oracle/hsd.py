"""HSD recursion (Alg. 1) and the generation loop around it.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Follows Alg. 1 in the paper's order: level 0 drafts T_0 tokens one at a time and
keeps each full distribution; an intermediate level idx repeatedly asks the
level below for a batch, verifies it (Alg. 2) and collects the verified tokens
until it holds at least T_idx of them, then returns ALL it collected (so the
level above may see more than T_idx tokens: Alg. 1 returns `tokens`, not a
prefix; the footnote to the definition of gamma in Sec. 3.3 notes the same);
the top level K does one such batch + verification.  Each recursive call
starts from empty lists, so what a lower level buffered beyond a rejection is
discarded.

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

    def run(self, idx, context):
        """HSD(idx, context) -> (tokens, probs)."""
        tokens, probs, count = [], [], 0
        if idx == 0:
            while count < (self.T[0] if self.K > 0 else 1):
                p = self.levels[0].next_dists(list(context) + tokens, 1)[0]
                self.passes[0] += 1
                call = self.calls[0]
                self.calls[0] += 1
                tokens.append(self.chooser.sample(0, call, 0, p, None))
                probs.append(p)
                count += 1
        elif idx == self.K:
            dt, dp = self.run(idx - 1, context)
            tokens, probs = self._verify(idx, dt, dp, context)
        else:
            while count < self.T[idx]:
                ctx = list(context) + tokens
                dt, dp = self.run(idx - 1, ctx)
                vt, vp = self._verify(idx, dt, dp, ctx)
                tokens.extend(vt)
                probs.extend(vp)
                count += len(vt)
            if self.truncate:
                tokens, probs = tokens[:self.T[idx]], probs[:self.T[idx]]
        return tokens, probs

    def generate(self, prompt, n_tokens):
        """Call HSD(K, context) until n_tokens are produced; the last round is cut at n_tokens.
        With a single level (K = 0) this is plain autoregressive sampling from that model."""
        out = []
        while len(out) < n_tokens:
            toks, _ = self.run(self.K, list(prompt) + out)
            out.extend(toks)
        return out[:n_tokens]
