"""Plain fp64 decoder with early exits: the language model M_i of Sec. 3.2.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper treats M_i(context) -> (t, p) as a black box and, for its
experiments, takes M_i to be the hidden state after layer i of one transformer
passed through an output head (Sec. 5.1; LayerSkip shares one head).  The
architecture itself comes from the workload description, not the paper:
pre-norm decoder, RMSNorm (eps inside the square root), rotary position
embedding on q and k (half-split pairing: dims j and j+hd/2 rotate together,
angle pos * base^(-2j/hd)), grouped-query causal attention with 1/sqrt(hd)
scaling, SwiGLU feed-forward, untied output head preceded by a final RMSNorm
that every exit shares.  Linear weights are stored [out_features, in_features].

Everything is the textbook definition in fp64: no blocking, no fusion.  The
KV cache is a flat array per layer; a pass over M new tokens must equal M
single-token passes and a from-scratch pass over the whole sequence (pinned in
tests/test_oracle_decoder.py against an independent torch fp64 formulation).
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Spec:
    n_layers: int
    d: int
    n_q: int
    n_kv: int
    hd: int
    ffn: int
    vocab: int
    rope_base: float = 10000.0
    eps: float = 1e-5


LAYER_KEYS = ("norm1", "wq", "wk", "wv", "wo", "norm2", "wg", "wu", "wd")


def rmsnorm(x, w, eps):
    return x * w / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)


def rope(x, positions, base):
    """x: [M, heads, hd]; rotate (x_j, x_{j+hd/2}) by angle pos * base^(-2j/hd)."""
    hd = x.shape[-1]
    half = hd // 2
    inv = base ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv[None, :]        # [M, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def softmax_rows(z):
    z = z - np.max(z, axis=-1, keepdims=True)
    e = np.exp(z)
    return e / np.sum(e, axis=-1, keepdims=True)


def distributions(logits, temperature):
    """Rows p = softmax(z / temperature) as fp32; temperature 0 gives the one-hot row at the
    lowest-index maximum of the fp32-rounded logits (the precision the library decides it in)."""
    z = np.asarray(logits, dtype=np.float64)
    if temperature == 0:
        z32 = z.astype(np.float32)
        out = np.zeros(z.shape, dtype=np.float32)
        out[np.arange(z.shape[0]), np.argmax(z32, axis=-1)] = 1.0
        return out
    return softmax_rows(z / temperature).astype(np.float32)


class Decoder:
    """One physical transformer; exits are prefixes of its layer stack."""

    def __init__(self, spec, weights, max_len):
        self.spec = spec
        f8 = lambda a: np.asarray(a, dtype=np.float64)
        self.embed = f8(weights["embed"])
        self.head = f8(weights["head"])
        self.norm_f = f8(weights["norm_f"])
        self.layers = [{k: f8(weights["layers"][i][k]) for k in LAYER_KEYS} for i in range(spec.n_layers)]
        s = spec
        self.K = np.zeros((s.n_layers, max_len, s.n_kv, s.hd))
        self.V = np.zeros((s.n_layers, max_len, s.n_kv, s.hd))
        self.cache_tokens = []                   # token ids the cache rows were computed from
        self.n_valid = [0] * s.n_layers          # per layer: rows [0, n_valid) match cache_tokens

    # -- plain forward over new tokens at positions pos0.., cache rows < pos0 must be valid --
    def _layer(self, j, x, pos0):
        s, w = self.spec, self.layers[j]
        M = x.shape[0]
        pos = np.arange(pos0, pos0 + M)
        n1 = rmsnorm(x, w["norm1"], s.eps)
        q = rope((n1 @ w["wq"].T).reshape(M, s.n_q, s.hd), pos, s.rope_base)
        k = rope((n1 @ w["wk"].T).reshape(M, s.n_kv, s.hd), pos, s.rope_base)
        v = (n1 @ w["wv"].T).reshape(M, s.n_kv, s.hd)
        self.K[j, pos0:pos0 + M] = k
        self.V[j, pos0:pos0 + M] = v
        group = s.n_q // s.n_kv
        att = np.zeros((M, s.n_q, s.hd))
        for i in range(M):
            L = pos0 + i + 1                     # causal: positions 0..pos0+i
            for h in range(s.n_q):
                g = h // group
                sc = self.K[j, :L, g] @ q[i, h] / np.sqrt(s.hd)
                p = softmax_rows(sc[None, :])[0]
                att[i, h] = p @ self.V[j, :L, g]
        h1 = x + att.reshape(M, s.n_q * s.hd) @ w["wo"].T
        n2 = rmsnorm(h1, w["norm2"], s.eps)
        gate = n2 @ w["wg"].T
        up = n2 @ w["wu"].T
        act = gate / (1.0 + np.exp(-gate)) * up
        return h1 + act @ w["wd"].T

    def forward(self, tokens, pos0, exit_layer):
        """Logits [M, V] (fp64) of the exit after `exit_layer` layers for `tokens` at pos0.."""
        x = self.embed[np.asarray(tokens, dtype=np.int64)]
        for j in range(exit_layer):
            x = self._layer(j, x, pos0)
        return rmsnorm(x, self.norm_f, self.spec.eps) @ self.head.T

    # -- cache bookkeeping by longest common prefix: semantics are cache-free --
    def next_logits(self, context, n_rows, exit_layer):
        """Logits of the last n_rows prefixes of `context`: row r is the next-token logits
        given context[: len-n_rows+1+r].  Re-uses cached rows whose tokens still match."""
        ctx = [int(t) for t in context]
        common = 0
        for a, b in zip(self.cache_tokens, ctx):
            if a != b:
                break
            common += 1
        start = min([common, len(ctx) - n_rows] + [self.n_valid[j] for j in range(exit_layer)])
        logits = self.forward(ctx[start:], start, exit_layer)
        for j in range(self.spec.n_layers):
            self.n_valid[j] = len(ctx) if j < exit_layer else min(self.n_valid[j], common)
        self.cache_tokens = ctx
        return logits[len(logits) - n_rows:]

    def reset(self):
        self.cache_tokens = []
        self.n_valid = [0] * self.spec.n_layers


class Level:
    """Hierarchy level = (decoder, exit layer, temperature, optional logit post-processing).
    `next_dists(context, n_rows)` returns the fp32 distribution rows of Alg. 2's verifier pass."""

    def __init__(self, decoder, exit_layer, temperature, logit_hook=None):
        self.decoder = decoder
        self.exit_layer = exit_layer
        self.temperature = temperature
        self.logit_hook = logit_hook
        self.last_logits = None
        self.min_top2_gap = float("inf")     # smallest gap between the two largest logits of any row seen

    def next_dists(self, context, n_rows):
        z = self.decoder.next_logits(context, n_rows, self.exit_layer)
        if self.logit_hook is not None:
            z = self.logit_hook(z, context, n_rows)
        self.last_logits = z
        top2 = np.partition(np.asarray(z, dtype=np.float64), -2, axis=-1)[:, -2:]
        self.min_top2_gap = min(self.min_top2_gap, float(np.min(top2[:, 1] - top2[:, 0])))
        return distributions(z, self.temperature)
