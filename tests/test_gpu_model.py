"""GPU parity of the decoder pass (all kernels assembled) against the fp64 oracle decoder."""
import numpy as np
import pytest

from paper_2510_19705_amd import inputs
from helpers import gpu_model, oracle_decoder, say

pytestmark = pytest.mark.gpu

# ragged on purpose: vocab not a multiple of 16, FFN a single odd multiple of 32, few heads
SMALL_F32 = dict(n_layers=3, d=96, n_q=6, n_kv=2, hd=32, ffn=160, vocab=777)
SMALL_BF16 = dict(n_layers=4, d=256, n_q=8, n_kv=2, hd=64, ffn=608, vocab=5000)
SMALL_BF16_MHA = dict(n_layers=2, d=256, n_q=2, n_kv=2, hd=128, ffn=512, vocab=1000)


def _tokens_dev(tok):
    import torch
    return torch.from_numpy(np.ascontiguousarray(tok, dtype=np.int32)).cuda()


def _run_passes(model, oracle, toks, schedule, exits):
    """schedule: list of (pos0, m, exit_index, n_logit_rows).  Yields (gpu logits, oracle logits)."""
    for pos0, m, e, nl in schedule:
        got = model.model_pass(_tokens_dev(toks[pos0:pos0 + m]), pos0, exits[e], nl).cpu().numpy()
        ref = oracle.forward([int(t) for t in toks[pos0:pos0 + m]], pos0, exits[e])[m - nl:]
        yield (pos0, m, exits[e], nl), got, ref


def test_pass_fp32_logits_rel_1e4():
    """fp32 storage: logits within 1e-4 relative (of the row's largest magnitude) of the oracle, over
    prefill chunks, a paged (permuted) cache, multi-token passes at different exits and rewrites of
    rejected positions."""
    shape = SMALL_F32
    w = inputs.make_weights(shape, seed=11, bf16=False)
    toks = inputs.make_prompt(shape["vocab"], 200, seed=12)
    model = gpu_model(shape, w, False, max_seq=256, max_rows=24)
    model.set_pages([2, 0, 3, 1])
    oracle = oracle_decoder(shape, w, 256)
    exits = (1, 2, 3)
    schedule = [(0, 24, 2, 0), (24, 24, 2, 3), (48, 17, 2, 17), (65, 1, 0, 1), (65, 1, 2, 1), (66, 5, 1, 5),
                (66, 7, 2, 7), (70, 24, 2, 24), (94, 24, 2, 1), (118, 24, 2, 0), (142, 6, 2, 6)]
    for tag, got, ref in _run_passes(model, oracle, toks, schedule, exits):
        if got.shape[0] == 0:
            continue
        err = np.abs(got - ref).max() / np.abs(ref).max()
        say("fp32 pass", tag, "rel err %.2e" % err)
        assert err < 1e-4, tag
    model.close()


@pytest.mark.parametrize("shape,rows_copy", [(SMALL_BF16, 2), (SMALL_BF16, 0), (SMALL_BF16_MHA, 2)],
                         ids=["gqa_hd64_rowcopies", "gqa_hd64", "mha_hd128_rowcopies"])
def test_pass_bf16_logits_abs_2e2(shape, rows_copy):
    """bf16 storage (MFMA GEMMs, MFMA attention over the tiled cache; with row copies the one-token passes
    go through the row kernel in the first layers): logits within 2e-2 absolute."""
    w = inputs.make_weights(shape, seed=21, bf16=True)
    toks = inputs.make_prompt(shape["vocab"], 330, seed=22)
    model = gpu_model(shape, w, True, max_seq=384, max_rows=64, rows_copy_layers=rows_copy)
    model.set_pages([5, 1, 4, 0, 3, 2])
    oracle = oracle_decoder(shape, w, 384)
    L = shape["n_layers"]
    exits = (1, L // 2, L)
    schedule = [(0, 64, 2, 0), (64, 64, 2, 2), (128, 33, 2, 33), (161, 1, 0, 1), (161, 1, 2, 1), (162, 6, 1, 6),
                (162, 9, 2, 9), (171, 64, 2, 0), (235, 64, 2, 5), (299, 17, 2, 17), (316, 2, 0, 2), (316, 2, 2, 2),
                (318, 1, 1, 1), (318, 4, 2, 4)]
    worst = 0.0
    for tag, got, ref in _run_passes(model, oracle, toks, schedule, exits):
        if got.shape[0] == 0:
            continue
        err = np.abs(got - ref).max()
        worst = max(worst, err)
        say("bf16 pass", tag, "abs err %.2e (|z| max %.2f)" % (err, np.abs(ref).max()))
        assert err < 2e-2, tag
    assert worst > 0                                      # bf16 rounding is visible: the path really is bf16
    model.close()


def test_pass_random_shapes_bf16():
    """Ten decoder shapes drawn at random (widths that are odd multiples of 32, one to four KV heads, grouped and
    plain attention, both head sizes, ragged vocabularies), each driven through a prefill chunk, one-token passes and
    multi-token passes of random sizes at random exits: bf16 logits within 2e-2 absolute of the oracle."""
    rng = np.random.default_rng(20251019)
    for trial in range(10):
        hd = int(rng.choice([64, 128]))
        n_kv = int(rng.choice([1, 2, 4]))
        n_q = n_kv * int(rng.choice([1, 2, 4]))
        L = int(rng.integers(1, 4))
        shape = dict(n_layers=L, d=32 * int(rng.integers(2, 17)), n_q=n_q, n_kv=n_kv, hd=hd,
                     ffn=32 * int(rng.integers(3, 33)), vocab=int(rng.integers(100, 6000)))
        say("shape", shape)
        w = inputs.make_weights(shape, seed=100 + trial, bf16=True)
        toks = inputs.make_prompt(shape["vocab"], 200, seed=200 + trial)
        model = gpu_model(shape, w, True, max_seq=256, max_rows=64, rows_copy_layers=int(rng.integers(0, L + 1)))
        oracle = oracle_decoder(shape, w, 256)
        pos = int(rng.integers(1, 65))
        schedule = [(0, pos, L - 1, 1)]
        for _ in range(5):
            m = int(rng.choice([1, 1, 2, int(rng.integers(3, 17)), int(rng.integers(17, 65))]))
            m = min(m, 200 - pos)
            e = int(rng.integers(0, L))
            # the cache of layers above an early exit is not filled by that pass: follow it with a full one
            schedule += [(pos, m, e, int(rng.integers(1, m + 1))), (pos, m, L - 1, m)]
            pos += int(rng.integers(0, m + 1))               # the next pass rewrites the positions after `pos`
        for tag, got, ref in _run_passes(model, oracle, toks, schedule, tuple(range(1, L + 1))):
            err = np.abs(got - ref).max()
            assert err < 2e-2, (shape, tag, err)
        model.close()


def test_pass_bf16_row_kernel_on_every_projection():
    """By default only the attention output (one token) and the FFN down projection (one or two tokens) take the
    row kernel; here q/k/v (RoPE + cache append epilogue) and three-token passes are sent through it as well."""
    from paper_2510_19705_amd import hsd
    shape = SMALL_BF16
    w = inputs.make_weights(shape, seed=41, bf16=True)
    toks = inputs.make_prompt(shape["vocab"], 100, seed=42)
    model = gpu_model(shape, w, True, max_seq=128, max_rows=64, rows_copy_layers=shape["n_layers"])
    model.set_tuning(gemv_max_m_qkv=3, gemv_max_m_o=3, gemv_max_m_down=3)          # this model only
    oracle = oracle_decoder(shape, w, 128)
    L = shape["n_layers"]
    schedule = [(0, 40, L - 1, 1), (40, 1, L - 1, 1), (41, 2, L - 1, 2), (43, 3, L - 1, 3), (46, 4, L - 1, 4), (50, 1, 0, 1), (50, 1, L - 1, 1)]
    for tag, got, ref in _run_passes(model, oracle, toks, schedule, tuple(range(1, L + 1))):
        err = np.abs(got - ref).max()
        say("row kernel everywhere", tag, "abs err %.2e" % err)
        assert err < 2e-2, tag
    model.close()


@pytest.mark.parametrize("max_groups", [0, 128], ids=["whole_tiles", "half_tiles"])
def test_pass_bf16_narrow_projection_schemes(max_groups):
    """The narrow projections (q/k/v, attention output, FFN down) of passes of few rows run with two workgroups per
    column group, each owning half of the columns of its tiles; switched off they keep whole tiles (FFN down then
    splits K over two workgroups).  Both against the oracle, 1 to 9 rows (the scheme applies up to 8)."""
    from paper_2510_19705_amd import hsd
    shape = dict(n_layers=2, d=512, n_q=8, n_kv=2, hd=64, ffn=8192, vocab=1000)       # down: K = 8192
    w = inputs.make_weights(shape, seed=31, bf16=True)
    toks = inputs.make_prompt(shape["vocab"], 120, seed=32)
    model = gpu_model(shape, w, True, max_seq=128, max_rows=64)
    model.set_tuning(halves_max_groups=max_groups)
    oracle = oracle_decoder(shape, w, 128)
    schedule = [(0, 50, 1, 1), (50, 1, 1, 1), (51, 3, 1, 3), (54, 8, 1, 8), (62, 9, 1, 9), (71, 5, 0, 5), (71, 5, 1, 5)]
    for tag, got, ref in _run_passes(model, oracle, toks, schedule, (1, 2)):
        err = np.abs(got - ref).max()
        say("narrow projections", "half tiles" if max_groups else "whole tiles", tag, "abs err %.2e" % err)
        assert err < 2e-2, tag
    model.close()


def test_pass_rejects_bad_arguments():
    shape = SMALL_F32
    w = inputs.make_weights(shape, seed=1, bf16=False)
    from paper_2510_19705_amd import hsd
    model = hsd.Model(shape, hsd.F32, 128, 8, inputs.ROPE_BASE, inputs.EPS)
    tok = _tokens_dev(np.zeros(8))
    with pytest.raises(hsd.HsdError) as e:                # weights not loaded yet
        model.model_pass(tok[:2], 0, 1, 1)
    assert e.value.code == -3
    model.load(w)
    for args, code in [((tok, 125, 1, 1), -2),            # positions beyond the KV capacity
                       ((tok[:2], 0, 4, 1), -1),          # exit layer out of range
                       ((tok[:2], 0, 1, 3), -1)]:         # more logit rows than tokens
        with pytest.raises(hsd.HsdError) as e:
            model.model_pass(*args)
        assert e.value.code == code, args
    import torch
    big = torch.zeros(9, dtype=torch.int32, device="cuda")
    with pytest.raises(hsd.HsdError) as e:
        model.model_pass(big, 0, 1, 1)                    # more rows than max_rows
    assert e.value.code == -2
    with pytest.raises(hsd.HsdError):
        model.set_pages([0, 0])
    model.close()


@pytest.mark.parametrize("name,shape,bf16,batch,m", [
    ("f32_3x4", SMALL_F32, False, 3, 4), ("f32_9x1", SMALL_F32, False, 9, 1),
    ("bf16_gqa_5x4", SMALL_BF16, True, 5, 4), ("bf16_gqa_16x4", SMALL_BF16, True, 16, 4), ("bf16_gqa_64x1", SMALL_BF16, True, 64, 1),
    ("bf16_mha_8x8", SMALL_BF16_MHA, True, 8, 8),
])
def test_pass_batch_matches_the_oracle_per_sequence(name, shape, bf16, batch, m):
    """A batch of sequences through hsd_model_pass_batch (per-sequence positions and page tables in the RoPE / KV
    append epilogue and in the attention; residual, SwiGLU, norms and head by row): sequences of different lengths,
    pages dealt out in a random order; the verify pass of m tokens per sequence against the oracle run on each
    sequence by itself, every logit.  fp32 1e-4 relative, bf16 2e-2 absolute."""
    import torch
    w = inputs.make_weights(shape, seed=61, bf16=bf16)
    L = shape["n_layers"]
    chunk = 64 // batch if 64 // batch >= 1 else 1
    chunk = max(1, min(chunk, 8))
    lens = [2 * chunk + (b * 3) % (chunk + 1) for b in range(batch)]        # cached positions before the verify pass
    pages_per_seq = (max(lens) + m + 63) // 64
    max_seq = ((batch * pages_per_seq + 1) * 64)
    rng = np.random.default_rng(7)
    toks = rng.integers(0, shape["vocab"], size=(batch, max(lens) + m), dtype=np.int32)
    model = gpu_model(shape, w, bf16, max_seq=max_seq, max_rows=64)
    table = rng.permutation(max_seq // 64)[:batch * pages_per_seq].reshape(batch, pages_per_seq)
    model.set_batch(batch, pages_per_seq, table)
    td = _tokens_dev(toks)
    # prefill: two passes of `chunk` tokens per sequence, then one whose start differs per sequence (tokens fed twice
    # rewrite the same K/V), so that the sequences end at different lengths
    for start in ([0] * batch, [chunk] * batch, [l - chunk for l in lens]):
        idx = torch.tensor([[s + i for i in range(chunk)] for s in start], device="cuda")
        model.model_pass_batch(torch.gather(td, 1, idx).contiguous(), start, L, with_logits=False)
    idx = torch.tensor([[l + i for i in range(m)] for l in lens], device="cuda")
    got = model.model_pass_batch(torch.gather(td, 1, idx).contiguous(), lens, L).cpu().numpy()
    oracle = oracle_decoder(shape, w, max(lens) + m + 1)
    worst = 0.0
    for b in range(batch):
        oracle.reset()
        ref = oracle.forward([int(t) for t in toks[b, :lens[b] + m]], 0, L)[lens[b]:]
        err = np.abs(got[b] - ref).max()
        err = err if bf16 else err / np.abs(ref).max()
        worst = max(worst, err)
        assert err < (2e-2 if bf16 else 1e-4), (name, b, err)
    say("batch pass", name, "lengths", lens[:6], "worst err %.2e" % worst)
    # an early exit of the same batch, and the error paths
    got2 = model.model_pass_batch(torch.gather(td, 1, idx).contiguous(), lens, 1).cpu().numpy()
    oracle.reset()
    ref2 = oracle.forward([int(t) for t in toks[0, :lens[0] + m]], 0, 1)[lens[0]:]
    e2 = np.abs(got2[0] - ref2).max()
    assert (e2 if bf16 else e2 / np.abs(ref2).max()) < (2e-2 if bf16 else 1e-4)
    from paper_2510_19705_amd import hsd
    with pytest.raises(hsd.HsdError):
        model.model_pass_batch(td[:, :m].contiguous(), [pages_per_seq * 64 - m + 1] * batch, L)     # beyond a sequence's pages
    with pytest.raises(hsd.HsdError):
        model.set_batch(batch, pages_per_seq, np.zeros((batch, pages_per_seq), dtype=np.int32))        # a page used twice
    model.set_batch(0)
    with pytest.raises(hsd.HsdError):
        model.model_pass_batch(td[:, :m].contiguous(), lens, L)                                        # no geometry
    model.close()
