"""Seeded synthetic inputs shared by the tests, the bench and the oracle's callers.

Holds no arithmetic of the method: only shapes, random weights, random prompts
and random probability rows.  The paper's workloads (summarisation prompts,
trained LayerSkip / Gemma2 checkpoints, Sec. 5.1) are not available offline, so
random-init models of the same shapes and uniform-random token ids stand in.

Weight recipe: embedding ~ N(0,1); every linear ~ N(0, 1/fan_in); the two
matrices that write into the residual stream (attention output and FFN down
projection) are additionally scaled by 0.1 so that early exits stay close to
the final hidden state; norm weights ~ 1 + 0.1 N(0,1); head ~ N(0, 1/d).  For
bf16 models every tensor is rounded once (round-to-nearest-even) and both the
library and the oracle receive the rounded values.
"""
import numpy as np

SHAPES = {
    # name: n_layers, d, n_q, n_kv, hd, ffn, vocab
    "tiny": dict(n_layers=8, d=256, n_q=4, n_kv=4, hd=64, ffn=1024, vocab=2048),
    "1b": dict(n_layers=16, d=2048, n_q=32, n_kv=8, hd=64, ffn=8192, vocab=32000),
    "125m": dict(n_layers=12, d=768, n_q=12, n_kv=12, hd=64, ffn=2048, vocab=32000),
    "7b": dict(n_layers=32, d=4096, n_q=32, n_kv=32, hd=128, ffn=11008, vocab=32000),
    "8b": dict(n_layers=32, d=4096, n_q=32, n_kv=8, hd=128, ffn=14336, vocab=128256),
    "70b": dict(n_layers=80, d=8192, n_q=64, n_kv=8, hd=128, ffn=28672, vocab=128256),
}
ROPE_BASE = 10000.0
EPS = 1e-5

LAYER_SHAPES = lambda s: {
    "norm1": (s["d"],),
    "wq": (s["n_q"] * s["hd"], s["d"]),
    "wk": (s["n_kv"] * s["hd"], s["d"]),
    "wv": (s["n_kv"] * s["hd"], s["d"]),
    "wo": (s["d"], s["n_q"] * s["hd"]),
    "norm2": (s["d"],),
    "wg": (s["ffn"], s["d"]),
    "wu": (s["ffn"], s["d"]),
    "wd": (s["d"], s["ffn"]),
}


def bf16_round(a):
    """Round fp32 values to the nearest bf16 (ties to even); returns fp32 holding bf16 values."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a):
    """The 16-bit patterns of values that are already bf16-representable."""
    return (np.ascontiguousarray(a, dtype=np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def make_weights(shape, seed, bf16):
    """Dict of fp32 arrays: embed [V,d], head [V,d], norm_f [d], layers[i][key]."""
    rng = np.random.default_rng(seed)
    fin = (lambda a: bf16_round(a)) if bf16 else (lambda a: a)

    def normal(sh, std):
        return fin((rng.standard_normal(sh, dtype=np.float32) * np.float32(std)))

    d = shape["d"]
    w = {"embed": normal((shape["vocab"], d), 1.0),
         "head": normal((shape["vocab"], d), d ** -0.5),
         "norm_f": fin(1.0 + 0.1 * rng.standard_normal(d, dtype=np.float32)),
         "layers": []}
    for _ in range(shape["n_layers"]):
        lw = {}
        for key, sh in LAYER_SHAPES(shape).items():
            if len(sh) == 1:
                lw[key] = fin(1.0 + 0.1 * rng.standard_normal(sh, dtype=np.float32))
            else:
                std = sh[1] ** -0.5 * (0.1 if key in ("wo", "wd") else 1.0)
                lw[key] = normal(sh, std)
        w["layers"].append(lw)
    return w


def make_prompt(vocab, n, seed):
    return np.random.default_rng(seed).integers(0, vocab, size=n, dtype=np.int32)


def make_prob_rows(vocab, t, seed, sigma=2.0, noise=1.0, one_hot=False):
    """Random target rows p [t+1, V], draft rows q [t, V] (fp32, each summing to ~1) and draft
    tokens x_i ~ q_i.  p = softmax(N(0, sigma^2) logits), q = softmax(the same logits + N(0, noise^2))."""
    rng = np.random.default_rng(seed)
    z = rng.standard_normal((t + 1, vocab)) * sigma
    zq = z[:t] + rng.standard_normal((t, vocab)) * noise

    def sm(a):
        if one_hot:
            o = np.zeros(a.shape, dtype=np.float32)
            o[np.arange(a.shape[0]), np.argmax(a, axis=-1)] = 1.0
            return o
        e = np.exp(a - a.max(axis=-1, keepdims=True))
        return (e / e.sum(axis=-1, keepdims=True)).astype(np.float32)

    p, q = sm(z), sm(zq)
    x = np.array([rng.choice(vocab, p=q[i].astype(np.float64) / q[i].astype(np.float64).sum())
                  for i in range(t)], dtype=np.int32)
    return p, q, x


def make_logit_rows(vocab, t, seed, sigma=2.0, noise=1.0):
    """Verifier logits z [t+1, V] (fp32), draft rows q [t, V] (fp32 probabilities of perturbed logits) and draft
    tokens x_i ~ q_i: the inputs of the fused softmax + Verify launch."""
    rng = np.random.default_rng(seed)
    z = (rng.standard_normal((t + 1, vocab)) * sigma).astype(np.float32)
    zq = z[:t].astype(np.float64) + rng.standard_normal((t, vocab)) * noise
    e = np.exp(zq - zq.max(axis=-1, keepdims=True)) if t else zq
    q = (e / e.sum(axis=-1, keepdims=True)).astype(np.float32) if t else zq.astype(np.float32)
    x = np.array([rng.choice(vocab, p=q[i].astype(np.float64) / q[i].astype(np.float64).sum())
                  for i in range(t)], dtype=np.int32)
    return z, q, x
