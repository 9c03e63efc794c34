"""Pins for oracle/decoder.py (CPU only): the numpy decoder against an independent torch fp64
formulation built from library routines, and its cache bookkeeping against cache-free evaluation."""
import numpy as np
import pytest
import scipy.special
import torch

from oracle import decoder
from paper_2510_19705_amd import inputs

SHAPE = dict(n_layers=3, d=48, n_q=6, n_kv=2, hd=8, ffn=80, vocab=37)


def _spec(shape):
    return decoder.Spec(shape["n_layers"], shape["d"], shape["n_q"], shape["n_kv"], shape["hd"], shape["ffn"],
                        shape["vocab"], inputs.ROPE_BASE, inputs.EPS)


def _torch_logits(shape, w, tokens, exit_layer):
    """Whole-sequence forward with torch library pieces: rms_norm, complex-multiplication RoPE,
    scaled_dot_product_attention with its causal flag, silu."""
    F = torch.nn.functional
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    n_q, n_kv, hd, d = shape["n_q"], shape["n_kv"], shape["hd"], shape["d"]
    S = len(tokens)
    x = t(w["embed"])[torch.tensor(tokens, dtype=torch.long)]
    pos = torch.arange(S, dtype=torch.float64)
    inv = inputs.ROPE_BASE ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    rot = torch.polar(torch.ones(S, hd // 2, dtype=torch.float64), pos[:, None] * inv[None, :])   # e^{i theta}

    def rope(a):                                   # a [S, H, hd]; pair (j, j + hd/2) as one complex number
        z = torch.complex(a[..., :hd // 2], a[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for j in range(exit_layer):
        lw = {k: t(v) for k, v in w["layers"][j].items()}
        n1 = F.rms_norm(x, (d,), lw["norm1"], eps=inputs.EPS)
        q = rope(F.linear(n1, lw["wq"]).view(S, n_q, hd)).transpose(0, 1)
        k = rope(F.linear(n1, lw["wk"]).view(S, n_kv, hd)).transpose(0, 1)
        v = F.linear(n1, lw["wv"]).view(S, n_kv, hd).transpose(0, 1)
        k = k.repeat_interleave(n_q // n_kv, dim=0)
        v = v.repeat_interleave(n_q // n_kv, dim=0)
        att = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
        x = x + F.linear(att.transpose(0, 1).reshape(S, n_q * hd), lw["wo"])
        n2 = F.rms_norm(x, (d,), lw["norm2"], eps=inputs.EPS)
        x = x + F.linear(F.silu(F.linear(n2, lw["wg"])) * F.linear(n2, lw["wu"]), lw["wd"])
    return F.linear(F.rms_norm(x, (d,), t(w["norm_f"]), eps=inputs.EPS), t(w["head"])).numpy()


@pytest.mark.parametrize("exit_layer", [1, 2, 3])
def test_forward_equals_torch_formulation(exit_layer):
    w = inputs.make_weights(SHAPE, seed=1, bf16=False)
    toks = [int(v) for v in inputs.make_prompt(SHAPE["vocab"], 11, seed=2)]
    dec = decoder.Decoder(_spec(SHAPE), w, max_len=32)
    got = dec.forward(toks, 0, exit_layer)
    ref = _torch_logits(SHAPE, w, toks, exit_layer)
    assert np.abs(got - ref).max() < 1e-10 * max(1.0, np.abs(ref).max())


def test_multi_token_pass_equals_single_token_passes():
    """Alg. 2's parallel verifier pass: scoring M tokens at once = M one-token passes = from scratch."""
    w = inputs.make_weights(SHAPE, seed=3, bf16=True)
    toks = [int(v) for v in inputs.make_prompt(SHAPE["vocab"], 13, seed=4)]
    a = decoder.Decoder(_spec(SHAPE), w, max_len=32)
    whole = a.forward(toks, 0, 3)
    b = decoder.Decoder(_spec(SHAPE), w, max_len=32)
    b.forward(toks[:7], 0, 3)
    chunk = b.forward(toks[7:], 7, 3)
    assert np.abs(chunk - whole[7:]).max() < 1e-12
    c = decoder.Decoder(_spec(SHAPE), w, max_len=32)
    rows = [c.forward(toks[i:i + 1], i, 3)[0] for i in range(13)]
    assert np.abs(np.stack(rows) - whole).max() < 1e-12


def test_cache_bookkeeping_is_semantics_free():
    """next_logits after appends, truncations, replaced tokens and exits of different depth always
    equals a fresh evaluation of the same context."""
    w = inputs.make_weights(SHAPE, seed=5, bf16=False)
    spec = _spec(SHAPE)
    dec = decoder.Decoder(spec, w, max_len=40)
    rng = np.random.default_rng(0)
    ctx = [int(v) for v in rng.integers(0, SHAPE["vocab"], 6)]
    for step in range(25):
        op = rng.integers(0, 3)
        if op == 0 or len(ctx) < 4:
            ctx = ctx + [int(v) for v in rng.integers(0, SHAPE["vocab"], rng.integers(1, 4))]
        elif op == 1:
            ctx = ctx[:len(ctx) - int(rng.integers(1, 3))]
        else:
            ctx = ctx[:len(ctx) - 2] + [int(rng.integers(0, SHAPE["vocab"]))]
        ctx = ctx[:38]
        e = int(rng.integers(1, 4))
        n_rows = int(rng.integers(1, min(4, len(ctx)) + 1))
        got = dec.next_logits(ctx, n_rows, e)
        fresh = decoder.Decoder(spec, w, max_len=40).forward(ctx, 0, e)[len(ctx) - n_rows:]
        assert np.abs(got - fresh).max() < 1e-11, step


def test_distributions():
    z = np.random.default_rng(1).standard_normal((4, 50)) * 3
    p = decoder.distributions(z, 0.7)
    assert p.dtype == np.float32
    assert np.abs(p - scipy.special.softmax(z / 0.7, axis=-1)).max() < 1e-7
    z[1, 7] = z[1, 30] = z[1].max() + 1.0        # tie: lowest index wins
    oh = decoder.distributions(z, 0)
    assert (oh.sum(axis=-1) == 1).all() and oh[1, 7] == 1.0
    assert (np.argmax(oh, axis=-1) == np.argmax(z.astype(np.float32), axis=-1)).all()


def test_bf16_rounding_of_inputs():
    a = np.array([1.0, 1.00390625, 1.005859375, 1.001953125, -3.14159, 65504.0, 1e-30], dtype=np.float32)
    r = inputs.bf16_round(a)
    ref = torch.tensor(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert (r == ref).all()
    assert (inputs.bf16_bits(r).astype(np.uint32) << 16).astype(np.uint32).view(np.float32).tolist() == r.tolist()
