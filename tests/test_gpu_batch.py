"""HSD over a batch of sequences in lockstep (hsd_batch_*): every sequence must come out as the oracle's Alg. 1 / 2
produce it alone (own prompt, own sampling seed), whatever the other sequences of the batch do."""
import numpy as np
import pytest

from oracle import decoder, hsd as ohsd, specsample
from paper_2510_19705_amd import inputs
from helpers import gpu_model, oracle_decoder, say

pytestmark = pytest.mark.gpu

TINY = inputs.SHAPES["tiny"]
EXITS = (2, 4, 8)
MAX_LEN = 192
# (prompt seed, prompt length, sampling seed): found with the oracle alone (python tests/scan_stream_seeds.py --batch:
# on 48 tokens, T = (4, 2)) for the margins asserted below; ragged prompt lengths
T1_SEQUENCES = [(2, 40, 220), (3, 24, 231), (4, 32, 240), (5, 40, 250), (6, 24, 264), (7, 32, 274)]
T0_SEQUENCES = [(10, 32, 1), (11, 40, 1), (13, 32, 1), (15, 24, 1), (21, 24, 1), (26, 40, 1)]


@pytest.fixture(scope="module")
def tiny():
    w = inputs.make_weights(TINY, seed=1, bf16=False)
    model = gpu_model(TINY, w, False, max_seq=6 * MAX_LEN, max_rows=64)
    yield w, model
    model.close()


def _oracle_stream(w, exits, T, temperature, pseed, n_prompt, seed, n):
    dec = oracle_decoder(TINY, w, n_prompt + n + 64)
    levels = [decoder.Level(dec, e, temperature) for e in exits]
    ch = specsample.PhiloxChooser(seed)
    o = ohsd.HSD(levels, T, ch)
    prompt = [int(t) for t in inputs.make_prompt(TINY["vocab"], n_prompt, seed=pseed)]
    ref = o.generate(prompt, n)
    if temperature == 0:
        assert min(l.min_top2_gap for l in levels) > 1.5e-3, (pseed, n_prompt)
    else:
        assert min(ch.accept_margins) > 3e-4 and min(ch.sample_margins) > 3e-6, (pseed, n_prompt, seed)
    return prompt, ref, o


@pytest.mark.parametrize("temperature,seqs", [(1.0, T1_SEQUENCES), (0.0, T0_SEQUENCES)], ids=["t1", "t0"])
@pytest.mark.parametrize("batch", [1, 3, 6])
def test_batch_streams_equal_the_oracle_per_sequence(tiny, temperature, seqs, batch):
    """Three-level hierarchy, T = (4, 2), fp32: 48 tokens of every sequence equal the oracle's stream of that sequence
    alone, and the summed acceptance counters equal the sum of the oracle's; the number of batched passes of a level is
    at least that of its busiest sequence and at most the sum over the sequences."""
    from paper_2510_19705_amd import hsd
    w, model = tiny
    T, n = (4, 2), 48
    runs = [_oracle_stream(w, EXITS, T, temperature, ps, npr, sd, n) for ps, npr, sd in seqs[:batch]]
    h = hsd.BatchHierarchy([(model, e) for e in EXITS], T, temperature, [s[2] for s in seqs[:batch]], MAX_LEN)
    h.prefill([r[0] for r in runs])
    got, st = h.generate(n)
    for b, (_, ref, _) in enumerate(runs):
        assert got[b].tolist() == ref, "sequence %d of %d" % (b, batch)
    for i in range(3):
        assert st.drafted[i] == sum(r[2].drafted[i] for r in runs) and st.accepted[i] == sum(r[2].accepted[i] for r in runs)
        assert max(r[2].passes[i] for r in runs) <= st.passes[i] <= sum(r[2].passes[i] for r in runs)
    say("batch %d at temperature %g: passes %s (alone: %s), tokens %d in %d rounds" % (
        batch, temperature, [st.passes[i] for i in range(3)], [[r[2].passes[i] for i in range(3)] for r in runs], st.tokens, st.rounds))
    # a second generation continues every sequence: equal to the oracle's next tokens
    more, _ = h.generate(8)
    for b, (prompt, ref, o) in enumerate(runs):
        assert h.sequence_length(b) >= len(prompt) + n + 8
    h.close()


def test_batch_plain_decoding_and_two_levels(tiny):
    """K = 0 (plain decoding of a batch: at temperature 0 the greedy continuations) and K = 1 (one drafter, T = 5)."""
    from paper_2510_19705_amd import hsd
    w, model = tiny
    n = 32
    runs = [_oracle_stream(w, (8,), (), 0.0, ps, npr, 1, n) for ps, npr, _ in T0_SEQUENCES[:4]]
    h = hsd.BatchHierarchy([(model, 8)], (), 0.0, [1, 2, 3, 4], MAX_LEN)
    h.prefill([r[0] for r in runs])
    got, st = h.generate(n)
    for b, (_, ref, _) in enumerate(runs):
        assert got[b].tolist() == ref
    assert st.passes[0] == n and st.tokens == 4 * n
    h.close()
    h = hsd.BatchHierarchy([(model, 2), (model, 8)], (5,), 0.0, [1, 2, 3, 4], MAX_LEN)
    h.prefill([r[0] for r in runs])
    got, st = h.generate(n)
    for b, (_, ref, _) in enumerate(runs):
        assert got[b].tolist() == ref                      # Thm 3.1 at temperature 0: the target's greedy stream
    assert st.accepted[1] > 0
    h.close()


def test_batch_bf16_emits_the_targets_greedy_tokens():
    """bf16 storage, a mid-sized network, temperature 0: a batch run cannot be bit-identical to single-sequence runs
    (other row counts select other kernels, and a near-tie may then fall the other way), so every emitted token is
    checked against the fp64 oracle's logits at the context the library itself produced: it must be the target's
    argmax up to twice the bf16 logit tolerance (Thm 3.1 at temperature 0), and most tokens must be the exact argmax."""
    from paper_2510_19705_amd import hsd
    shape = dict(n_layers=4, d=256, n_q=8, n_kv=2, hd=64, ffn=608, vocab=5000)
    w = inputs.make_weights(shape, seed=61, bf16=True)
    model = gpu_model(shape, w, True, max_seq=4 * 128, max_rows=64)
    n, B = 24, 4
    prompts = [[int(t) for t in inputs.make_prompt(shape["vocab"], 20 + 4 * b, seed=70 + b)] for b in range(B)]
    h = hsd.BatchHierarchy([(model, 1), (model, 2), (model, 4)], (3, 2), 0.0, list(range(B)), 128)
    h.prefill(prompts)
    got, st = h.generate(n)
    exact = 0
    for b in range(B):
        dec = oracle_decoder(shape, w, 128)
        z = dec.forward(prompts[b] + got[b].tolist(), 0, 4)
        for i in range(n):
            row = z[len(prompts[b]) - 1 + i]
            assert row[got[b, i]] >= row.max() - 4e-2, (b, i)
            exact += int(got[b, i] == int(np.argmax(row)))
    say("bf16 batch: %d of %d tokens are the oracle's exact argmax; accepted %s of %s" % (
        exact, B * n, [st.accepted[i] for i in range(3)], [st.drafted[i] for i in range(3)]))
    assert exact >= 0.9 * B * n
    assert st.accepted[1] > 0 and st.accepted[2] > 0
    h.close()
    model.close()


def test_batch_of_twenty_sequences():
    """More sequences than one launch of the batched sampler takes (16): twenty short sequences, one drafter with T = 1,
    temperature 0; every sequence is the target's greedy continuation (the oracle's top-2 gap is asserted per prompt,
    prompts that do not have it are replaced by the next seed)."""
    from paper_2510_19705_amd import hsd
    w = inputs.make_weights(TINY, seed=1, bf16=False)
    model = gpu_model(TINY, w, False, max_seq=20 * 128, max_rows=64)
    n, prompts, refs, seed = 12, [], [], 100
    while len(prompts) < 20:
        dec = oracle_decoder(TINY, w, 64)
        lvl = decoder.Level(dec, 8, 0.0)
        prompt = [int(t) for t in inputs.make_prompt(TINY["vocab"], 8 + seed % 5, seed=seed)]
        ref = ohsd.HSD([lvl], (), specsample.PhiloxChooser(1)).generate(prompt, n)
        seed += 1
        if lvl.min_top2_gap > 1.5e-3:
            prompts.append(prompt)
            refs.append(ref)
    h = hsd.BatchHierarchy([(model, 2), (model, 8)], (1,), 0.0, list(range(20)), 128)
    h.prefill(prompts)
    got, st = h.generate(n)
    for b in range(20):
        assert got[b].tolist() == refs[b], b
    assert st.tokens >= 20 * n and st.passes[1] <= n
    h.close()
    model.close()


def test_batch_vocabulary_above_the_fused_sampler_limit():
    """Vocabulary 33001: the sampler of every sequence is softmax + accept / resample as separate launches, their
    results copied back per sequence.  Temperature 0, three ragged prompts (chosen with the oracle alone for a top-2
    gap above 1.5e-3 on 24 tokens, T = (3, 2)): every sequence is the oracle's greedy stream."""
    from paper_2510_19705_amd import hsd
    shape = dict(n_layers=4, d=128, n_q=2, n_kv=2, hd=64, ffn=256, vocab=33001)
    w = inputs.make_weights(shape, seed=71, bf16=False)
    model = gpu_model(shape, w, False, max_seq=3 * 128, max_rows=64)
    n, seqs = 24, [(30, 20), (33, 20), (34, 24)]
    prompts, refs = [], []
    for pseed, npr in seqs:
        dec = oracle_decoder(shape, w, 128)
        levels = [decoder.Level(dec, e, 0.0) for e in (1, 2, 4)]
        prompt = [int(t) for t in inputs.make_prompt(shape["vocab"], npr, seed=pseed)]
        refs.append(ohsd.HSD(levels, (3, 2), specsample.PhiloxChooser(1)).generate(prompt, n))
        assert min(l.min_top2_gap for l in levels) > 1.5e-3, pseed
        prompts.append(prompt)
    h = hsd.BatchHierarchy([(model, 1), (model, 2), (model, 4)], (3, 2), 0.0, [1, 2, 3], 128)
    h.prefill(prompts)
    got, st = h.generate(n)
    for b in range(3):
        assert got[b].tolist() == refs[b], b
    assert st.accepted[1] > 0 and st.accepted[2] > 0
    h.close()
    model.close()


def test_batch_error_paths(tiny):
    from paper_2510_19705_amd import hsd
    _, model = tiny
    with pytest.raises(hsd.HsdError):                       # 6 sequences x 192 positions fit, 7 do not
        hsd.BatchHierarchy([(model, 2), (model, 8)], (4,), 1.0, list(range(7)), MAX_LEN)
    with pytest.raises(hsd.HsdError):                       # 6 x (40 drafts + 2) rows do not fit a pass
        hsd.BatchHierarchy([(model, 2), (model, 8)], (40,), 1.0, list(range(6)), MAX_LEN)
    with pytest.raises(hsd.HsdError):
        hsd.BatchHierarchy([(model, 2), (model, 8)], (4,), 1.0, [1, 2], 100)       # not a multiple of the page size
    h = hsd.BatchHierarchy([(model, 2), (model, 8)], (4,), 1.0, [1, 2], MAX_LEN)
    with pytest.raises(hsd.HsdError):
        h.generate(4)                                       # nothing prefilled
    h.prefill([[1, 2, 3], [4, 5, 6, 7]])
    with pytest.raises(hsd.HsdError):
        h.generate(MAX_LEN)                                 # does not fit
    with pytest.raises(hsd.HsdError):
        h.prefill([[1, 2, 3], [TINY["vocab"], 5]])          # token outside the vocabulary
    out, _ = h.generate(4)
    assert out.shape == (2, 4)
    h.close()
