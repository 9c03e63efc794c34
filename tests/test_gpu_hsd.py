"""GPU end-to-end parity of draft / verify / the HSD round driver against the oracle's Alg. 1/2."""
import numpy as np
import pytest

from oracle import decoder, hsd as ohsd, specsample
from paper_2510_19705_amd import inputs
from helpers import gpu_model, oracle_decoder, say

pytestmark = pytest.mark.gpu

TINY = inputs.SHAPES["tiny"]          # the smallest workload: 8 layers, d 256, 4 heads x 64, FFN 1024, vocab 2048
TINY_EXITS = (2, 4, 8)
SEED = 20251019


@pytest.fixture(scope="module")
def tiny():
    w = inputs.make_weights(TINY, seed=1, bf16=False)
    prompt = inputs.make_prompt(TINY["vocab"], 32, seed=2)
    model = gpu_model(TINY, w, False, max_seq=256, max_rows=16)
    yield w, prompt, model
    model.close()


def _oracle_levels(w, shape, exits, temperature, max_len=256):
    dec = oracle_decoder(shape, w, max_len)
    return [decoder.Level(dec, e, temperature) for e in exits]


def _gpu_hier(model, exits, T, temperature, seed=SEED):
    from paper_2510_19705_amd import hsd
    return hsd.Hierarchy([(model, e) for e in exits], T, temperature, seed)


@pytest.mark.parametrize("T", [(4, 2), (2, 4)])
def test_tiny_temperature0_stream_bit_exact(tiny, T):
    """Smallest workload, fp32, temperature 0: the 64 generated tokens equal the oracle's HSD stream and
    plain greedy decoding of the target.  The oracle's smallest top-2 logit gap must dwarf the fp32
    error bound, otherwise the comparison would be ill-posed (it is asserted, not assumed)."""
    w, _, model = tiny
    prompt = inputs.make_prompt(TINY["vocab"], 32, seed=10)     # prompt chosen (with the oracle alone) for a wide gap
    levels = _oracle_levels(w, TINY, TINY_EXITS, 0.0)
    o = ohsd.HSD(levels, T, specsample.PhiloxChooser(SEED))
    ref = o.generate([int(t) for t in prompt], 64)
    gap = min(l.min_top2_gap for l in levels)
    say("oracle min top-2 gap", gap)
    assert gap > 1.5e-3                                          # fp32 logit error is ~1e-5
    greedy = ohsd.HSD(_oracle_levels(w, TINY, (8,), 0.0), (), specsample.PhiloxChooser(1)).generate([int(t) for t in prompt], 64)
    assert ref == greedy
    h = _gpu_hier(model, TINY_EXITS, T, 0.0)
    h.prefill(prompt)
    got, st = h.generate(64)
    assert got.tolist() == ref
    assert [st.passes[i] for i in range(3)] == o.passes
    assert [st.drafted[i] for i in range(3)] == o.drafted and [st.accepted[i] for i in range(3)] == o.accepted
    h.close()
    # plain autoregressive decoding through the same library (one level): same stream
    ar = _gpu_hier(model, (8,), (), 0.0)
    ar.prefill(prompt)
    assert ar.generate(64)[0].tolist() == ref
    ar.close()


def test_temperature0_random_hierarchies(tiny):
    """At temperature 0 every hierarchy must emit the target's greedy continuation (Thm 3.1 with one-hot
    distributions), whatever its exits and T: sixteen hierarchies drawn at random (two to five levels, T of 1 to 5)
    against one greedy decode of the oracle, whose smallest top-2 gap is asserted to dwarf the fp32 error."""
    w, _, model = tiny
    prompt = inputs.make_prompt(TINY["vocab"], 32, seed=10)
    target = _oracle_levels(w, TINY, (8,), 0.0)
    ref = ohsd.HSD(target, (), specsample.PhiloxChooser(1)).generate([int(t) for t in prompt], 48)
    assert target[0].min_top2_gap > 1.5e-3
    rng = np.random.default_rng(4711)
    for trial in range(16):
        n_lower = int(rng.integers(1, 5))
        exits = tuple(sorted(rng.choice(np.arange(1, 8), size=n_lower, replace=False).tolist())) + (8,)
        T = tuple(int(t) for t in rng.integers(1, 6, size=n_lower))
        while sum(T) > 12:                                        # the verifier's pass takes at most 16 rows here
            T = tuple(max(1, t - 1) for t in T)
        say("hierarchy", exits, T)
        h = _gpu_hier(model, exits, T, 0.0, seed=SEED + trial)
        h.prefill(prompt)
        got, st = h.generate(48)
        assert got.tolist() == ref, (exits, T)
        assert sum(st.passes[i] for i in range(len(exits))) > 0
        h.close()


@pytest.fixture(params=["fused_sampler", "two_launch_sampler"])
def sampler_path(request):
    """The driver's two ways from logits to (n, token): the fused launch (vocabularies up to 32768) and softmax +
    accept/resample as two launches (larger vocabularies), the latter forced on the small vocabulary through the
    hierarchy's own settings.  Yields the settings to apply to a hierarchy."""
    return {} if request.param == "fused_sampler" else {"fused_sampler_max_v": 0}


@pytest.mark.parametrize("T,seed", [((4, 2), 104), ((3, 5), 100)])
def test_tiny_temperature1_stream(tiny, T, seed, sampler_path):
    """Temperature 1: same Philox stream on both sides.  Every accept test and every draw of the oracle
    run keeps a margin (asserted) far above the fp32 differences between the two softmaxes, so the
    streams, the accepted counts and the pass counts must be identical.  (A rounding-level change of a row
    moves a draw's interval ends by ~1e-7 of the total mass; the seeds were picked, with the oracle
    alone, so that no draw of the run lands closer than 3e-6 to an end.)"""
    w, prompt, model = tiny
    levels = _oracle_levels(w, TINY, TINY_EXITS, 1.0)
    ch = specsample.PhiloxChooser(seed)
    o = ohsd.HSD(levels, T, ch)
    ref = o.generate([int(t) for t in prompt], 64)
    say("oracle margins: accept %.2e sample %.2e" % (min(ch.accept_margins), min(ch.sample_margins)))
    assert min(ch.accept_margins) > 3e-4 and min(ch.sample_margins) > 3e-6
    h = _gpu_hier(model, TINY_EXITS, T, 1.0, seed=seed)
    h.set_tuning(**sampler_path)
    h.prefill(prompt)
    got, st = h.generate(64)
    assert got.tolist() == ref
    assert [st.drafted[i] for i in range(3)] == o.drafted and [st.accepted[i] for i in range(3)] == o.accepted
    assert [st.passes[i] for i in range(3)] == o.passes
    say("acceptance", [st.accepted[i] / max(1, st.drafted[i]) for i in (1, 2)], "rounds", st.rounds)
    h.close()


def test_temperature1_random_hierarchies(tiny):
    """Temperature 1, hierarchies, T and seeds drawn at random: wherever the oracle's run keeps the margins of the
    fixed-seed test above (decided by the oracle alone), stream, counts and passes must be identical; runs with a
    marginal decision are skipped and counted, and most runs must qualify."""
    w, prompt, model = tiny
    rng = np.random.default_rng(1234)
    compared = 0
    for trial in range(16):
        n_lower = int(rng.integers(1, 4))
        exits = tuple(sorted(rng.choice(np.arange(1, 8), size=n_lower, replace=False).tolist())) + (8,)
        T = tuple(int(t) for t in rng.integers(1, 5, size=n_lower))
        seed = 7000 + trial
        levels = _oracle_levels(w, TINY, exits, 1.0)
        ch = specsample.PhiloxChooser(seed)
        o = ohsd.HSD(levels, T, ch)
        ref = o.generate([int(t) for t in prompt], 40)
        wide = min(ch.accept_margins, default=1.0) > 3e-4 and min(ch.sample_margins) > 3e-6
        say("hierarchy", exits, T, "seed", seed, "margins wide" if wide else "marginal: skipped")
        if not wide:
            continue
        h = _gpu_hier(model, exits, T, 1.0, seed=seed)
        h.prefill(prompt)
        got, st = h.generate(40)
        n = len(exits)
        assert got.tolist() == ref, (exits, T, seed)
        assert [st.drafted[i] for i in range(n)] == o.drafted and [st.accepted[i] for i in range(n)] == o.accepted
        assert [st.passes[i] for i in range(n)] == o.passes
        h.close()
        compared += 1
    assert compared >= 8, compared


def test_draft_and_verify_calls(tiny):
    """The two building blocks: draft(k) rows and tokens, verify rows p_1..p_{n+1} and output tokens,
    each against the oracle (distribution rows by tolerance, tokens exactly)."""
    w, prompt, model = tiny
    levels = _oracle_levels(w, TINY, TINY_EXITS, 1.0)
    ch = specsample.PhiloxChooser(SEED)
    ctx = [int(t) for t in prompt]
    h = _gpu_hier(model, TINY_EXITS, (4, 2), 1.0)
    h.prefill(prompt)
    for rnd in range(3):
        # oracle: level 0 drafts 4 tokens, level 1 verifies them
        o = ohsd.HSD(levels, (4, 2), ch)
        o.calls = [4 * rnd, rnd, 0]
        dt, dq = o.run(0, ctx)
        vt, vp = o._verify(1, dt, dq, ctx)
        toks, q = h.draft(4)
        assert toks.tolist() == dt
        assert np.abs(q.cpu().numpy() - np.stack(dq)).max() < 1e-6
        out, p = h.verify(1, None, q, 4)
        assert out.tolist() == vt
        assert p.shape[0] == len(vt) and np.abs(p.cpu().numpy() - np.stack(vp)).max() < 1e-6
        ctx = ctx + vt
        assert h.sequence_length() == len(ctx)
    h.close()


def test_verify_with_host_drafts(tiny):
    """verify(level, drafted tokens, draft probs) with drafts supplied by the caller (here: the oracle's
    level-0 drafts and rows), as the boundary states it."""
    import torch
    w, prompt, model = tiny
    levels = _oracle_levels(w, TINY, TINY_EXITS, 1.0)
    ch = specsample.PhiloxChooser(7)
    ctx = [int(t) for t in prompt]
    o = ohsd.HSD(levels, (3, 2), ch)
    dt, dq = o.run(0, ctx)
    vt, vp = o._verify(2, dt, dq, ctx)                     # target verifies level-0 drafts directly
    h = _gpu_hier(model, TINY_EXITS, (3, 2), 1.0, seed=7)
    h.prefill(prompt)
    q = torch.from_numpy(np.stack(dq)).cuda()
    out, p = h.verify(2, dt, q, 3)
    assert out.tolist() == vt
    assert np.abs(p.cpu().numpy() - np.stack(vp)).max() < 1e-6
    h.close()


def test_rewind_repeats_the_generation(tiny):
    w, prompt, model = tiny
    h = _gpu_hier(model, TINY_EXITS, (4, 2), 1.0)
    h.prefill(prompt)
    a, _ = h.generate(40)
    h.rewind(len(prompt))
    b, _ = h.generate(40)
    assert a.tolist() == b.tolist()
    h.close()


def test_driver_error_paths(tiny):
    from paper_2510_19705_amd import hsd
    import torch
    w, prompt, model = tiny
    with pytest.raises(hsd.HsdError):                      # T_i >= 1
        _gpu_hier(model, TINY_EXITS, (4, 0), 1.0)
    with pytest.raises(hsd.HsdError) as e:                 # a verify pass of 15+4 drafts + 1 exceeds 16 rows
        _gpu_hier(model, TINY_EXITS, (15, 4), 1.0)
    assert e.value.code == -2
    with pytest.raises(hsd.HsdError):                      # exit layer out of range
        _gpu_hier(model, (2, 4, 9), (4, 2), 1.0)
    other = hsd.Model(dict(TINY, vocab=1000, n_layers=1), hsd.F32, 128, 8)
    with pytest.raises(hsd.HsdError) as e:                 # all models must share the vocabulary (Sec. 2)
        hsd.Hierarchy([(other, 1), (model, 8)], (2,), 1.0, 1)
    assert b"vocabulary" in hsd.lib.hsd_last_error()
    other.close()
    h = _gpu_hier(model, TINY_EXITS, (4, 2), 1.0)
    with pytest.raises(hsd.HsdError) as e:                 # nothing prefilled yet
        h.generate(4)
    assert e.value.code == -3
    with pytest.raises(hsd.HsdError):                      # token id outside the vocabulary
        h.prefill([1, 2, TINY["vocab"]])
    h.prefill(prompt)
    q = torch.zeros((4, TINY["vocab"]), device="cuda")
    with pytest.raises(hsd.HsdError):                      # level 0 only drafts
        h.verify(0, [1, 2], q, 2)
    with pytest.raises(hsd.HsdError):                      # level out of range
        h.verify(3, [1, 2], q, 2)
    with pytest.raises(hsd.HsdError):                      # more drafts than T_0
        h.draft(5)
    with pytest.raises(hsd.HsdError) as e:                 # only the lowest level drafts autoregressively (Alg. 1)
        h.draft(2, level=1)
    assert e.value.code == -1
    with pytest.raises(hsd.HsdError):                      # draft id outside the vocabulary
        h.verify(1, [1, -5], q, 2)
    h.close()
    big = _gpu_hier(model, TINY_EXITS, (4, 2), 0.0)
    big.prefill(inputs.make_prompt(TINY["vocab"], 250, seed=3))
    with pytest.raises(hsd.HsdError) as e:                 # KV capacity (256 tokens) exceeded
        big.generate(32)
    assert e.value.code == -2
    big.close()


def test_independent_models_in_one_hierarchy():
    """Levels that are different networks (Sec. 3.2: models sharing only the vocabulary): a small independent
    drafter under an early exit and the full stack of the second network.  Separate KV caches, separate validity
    bookkeeping.  Temperature 0 and 1 streams, pass and acceptance counts against the oracle (prompt / seed chosen
    with the oracle alone for the asserted margins)."""
    from paper_2510_19705_amd import hsd
    small = dict(n_layers=2, d=128, n_q=2, n_kv=1, hd=64, ffn=384, vocab=TINY["vocab"])
    wa = inputs.make_weights(small, seed=51, bf16=False)
    wb = inputs.make_weights(TINY, seed=1, bf16=False)
    ma = gpu_model(small, wa, False, max_seq=256, max_rows=16)
    mb = gpu_model(TINY, wb, False, max_seq=256, max_rows=16)
    da, db = oracle_decoder(small, wa, 256), oracle_decoder(TINY, wb, 256)
    T = (3, 2)
    for temperature, pseed, seed in [(0.0, 73, 1), (1.0, 2, 305)]:
        prompt = inputs.make_prompt(TINY["vocab"], 32, seed=pseed)
        da.reset()
        db.reset()
        levels = [decoder.Level(da, 2, temperature), decoder.Level(db, 4, temperature), decoder.Level(db, 8, temperature)]
        ch = specsample.PhiloxChooser(seed)
        o = ohsd.HSD(levels, T, ch)
        ref = o.generate([int(t) for t in prompt], 48)
        if temperature == 0:
            assert min(l.min_top2_gap for l in levels) > 1.5e-3
        else:
            assert min(ch.accept_margins) > 3e-4 and min(ch.sample_margins) > 3e-6
        h = hsd.Hierarchy([(ma, 2), (mb, 4), (mb, 8)], T, temperature, seed)
        h.prefill(prompt)
        got, st = h.generate(48)
        assert got.tolist() == ref, temperature
        assert [st.passes[i] for i in range(3)] == o.passes
        assert [st.drafted[i] for i in range(3)] == o.drafted and [st.accepted[i] for i in range(3)] == o.accepted
        say("independent models, temperature", temperature, "accepted", o.accepted, "of", o.drafted)
        h.close()
    # different vocabularies are refused
    other = dict(small, vocab=1000)
    mc = gpu_model(other, inputs.make_weights(other, seed=3, bf16=False), False, max_seq=64, max_rows=8)
    with pytest.raises(hsd.HsdError) as e:
        hsd.Hierarchy([(mc, 2), (mb, 8)], (2,), 1.0, 1)
    assert e.value.code == -1
    for m in (ma, mb, mc):
        m.close()


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
def test_token_embedded_by_the_sampler_changes_nothing(bf16):
    """The fused sampler leaves the token it emits embedded for the one-token pass that follows; with that switched
    off the embedding kernel does it.  Same tokens, same counters (bf16: the row's sum of squares is accumulated in
    the same order on both routes, so even the bits agree)."""
    from paper_2510_19705_amd import hsd
    shape = dict(n_layers=4, d=256, n_q=8, n_kv=2, hd=64, ffn=608, vocab=5000)
    w = inputs.make_weights(shape, seed=61, bf16=bf16)
    prompt = inputs.make_prompt(shape["vocab"], 40, seed=62)
    model = gpu_model(shape, w, bf16, max_seq=192, max_rows=16, rows_copy_layers=2 if bf16 else 0)
    runs = []
    for pre in (1, 0):
        h = hsd.Hierarchy([(model, 1), (model, 2), (model, 4)], (3, 2), 1.0, 77)
        h.set_tuning(preembed=pre)
        h.prefill(prompt)
        toks, st = h.generate(60)
        d = h.draft(2)                                  # explicit draft calls go the same way
        runs.append((toks.tolist(), [st.passes[i] for i in range(3)], [st.accepted[i] for i in range(3)], d[0].tolist()))
        h.close()
    assert runs[0] == runs[1]
    model.close()


@pytest.mark.parametrize("mode,seed", [("truncate", 502), ("coin", 501), ("both", 500)])
def test_ablation_modes_follow_the_oracle(tiny, mode, seed):
    """The switches of the appendix on HSD's assumptions: coin-flip acceptances (same Philox words, fixed
    probability per level) and the exactly-T variant of Alg. 1.  Streams, pass counts, accepted / tested counters
    equal the oracle's (seeds chosen with the oracle alone for the asserted margins)."""
    from paper_2510_19705_amd import hsd
    w, prompt, model = tiny
    T, coin = (3, 2), [0.0, 0.8, 0.6]
    levels = _oracle_levels(w, TINY, TINY_EXITS, 1.0)
    ch = specsample.IIDChooser(seed, coin) if mode != "truncate" else specsample.PhiloxChooser(seed)
    o = ohsd.HSD(levels, T, ch, truncate=(mode != "coin"))
    ref = o.generate([int(t) for t in prompt], 64)
    assert min(ch.accept_margins + [1.0]) > 3e-4 and min(ch.sample_margins) > 3e-6
    h = _gpu_hier(model, TINY_EXITS, T, 1.0, seed=seed)
    h.set_ablation(coin if mode != "truncate" else None, exactly_T=(mode != "coin"))
    h.prefill(prompt)
    got, st = h.generate(64)
    assert got.tolist() == ref
    assert [st.passes[i] for i in range(3)] == o.passes
    assert [st.accepted[i] for i in range(3)] == o.accepted and [st.tested[i] for i in range(3)] == o.tested
    assert [st.drafted[i] for i in range(3)] == o.drafted
    if mode != "coin":
        assert st.drafted[2] == 2 * st.passes[2]                 # the top level always sees exactly T_1 drafts
    cost = [1.0, 2.5, 7.0]
    assert hsd.stats_cost(st, cost) == sum(p * c for p, c in zip(o.passes, cost))
    # back to the real rule: the plain stream of this seed again
    h.set_ablation(None, False)
    h.rewind(len(prompt))
    levels = _oracle_levels(w, TINY, TINY_EXITS, 1.0)
    ch2 = specsample.PhiloxChooser(seed)
    ref2 = ohsd.HSD(levels, T, ch2).generate([int(t) for t in prompt], 24)
    if min(ch2.accept_margins) > 3e-4 and min(ch2.sample_margins) > 3e-6:
        assert h.generate(24)[0].tolist() == ref2
    with pytest.raises(hsd.HsdError):
        h.set_ablation([0.0, 1.5, 0.5])
    h.close()


def test_polling_and_stream_wait_agree(tiny):
    """The driver learns each Verify's result by polling the sampler's sequence number in pinned memory; with that
    switched off it waits for the stream.  Same stream of tokens and counters, over many verifies in a row."""
    from paper_2510_19705_amd import hsd
    _, prompt, model = tiny
    runs = []
    for poll in (1, 0, 1):
        h = _gpu_hier(model, TINY_EXITS, (2, 1), 1.0, seed=9)
        h.set_tuning(poll_mailbox=poll)
        h.prefill(prompt)
        toks, st = h.generate(150)
        runs.append((toks.tolist(), [st.passes[i] for i in range(3)], [st.accepted[i] for i in range(3)]))
        h.close()
    assert runs[0] == runs[1] == runs[2]


@pytest.mark.parametrize("name,exits,T,n,t0_prompt,t1_seed", [
    ("eight_levels", (1, 2, 3, 4, 5, 6, 7, 8), (2, 1, 1, 1, 1, 1, 1), 40, 11, 801),
    ("forty_drafts", (2, 8), (40,), 90, 12, 811)])
def test_largest_hierarchies(name, exits, T, n, t0_prompt, t1_seed):
    """The most levels the library takes (8) and verify passes of 41 rows (40 drafts + bonus row), against the oracle
    at temperature 0 and 1; prompts / seeds chosen with the oracle alone for the asserted margins."""
    w = inputs.make_weights(TINY, seed=1, bf16=False)
    model = gpu_model(TINY, w, False, max_seq=256, max_rows=64)
    for temperature, pseed, seed in ((0.0, t0_prompt, 1), (1.0, 2, t1_seed)):
        prompt = inputs.make_prompt(TINY["vocab"], 32, seed=pseed)
        levels = _oracle_levels(w, TINY, exits, temperature)
        ch = specsample.PhiloxChooser(seed)
        o = ohsd.HSD(levels, T, ch)
        ref = o.generate([int(t) for t in prompt], n)
        if temperature == 0:
            assert min(l.min_top2_gap for l in levels) > 1e-3
        else:
            assert min(ch.accept_margins) > 3e-4 and min(ch.sample_margins) > 3e-6
        h = _gpu_hier(model, exits, T, temperature, seed=seed)
        h.prefill(prompt)
        got, st = h.generate(n)
        assert got.tolist() == ref, (name, temperature)
        k = len(exits)
        assert [st.passes[i] for i in range(k)] == o.passes and [st.accepted[i] for i in range(k)] == o.accepted
        say(name, "temperature", temperature, "accepted", o.accepted, "of", o.drafted)
        h.close()
    model.close()


def test_sequence_up_to_the_last_cache_position():
    """Generation may fill the KV capacity exactly; one token more is refused with HSD_ECAPACITY and leaves the
    hierarchy usable (rewind + generate again gives the same tokens)."""
    from paper_2510_19705_amd import hsd
    w = inputs.make_weights(TINY, seed=1, bf16=False)
    model = gpu_model(TINY, w, False, max_seq=128, max_rows=16)
    prompt = inputs.make_prompt(TINY["vocab"], 100, seed=3)
    h = _gpu_hier(model, TINY_EXITS, (3, 2), 1.0, seed=5)
    h.prefill(prompt)
    with pytest.raises(hsd.HsdError) as e:
        h.generate(200)                                      # runs into the capacity of 128 positions
    assert e.value.code == -2
    full = h.sequence_length()
    assert 120 <= full <= 128
    h.rewind(100)
    a, _ = h.generate(16)
    h.rewind(100)
    b, _ = h.generate(16)
    assert a.tolist() == b.tolist()
    h.close()
    model.close()


@pytest.mark.parametrize("vocab,wseed,cases", [
    (33001, 71, ((0.0, 30, 1, 32), (1.0, 2, 911, 24))),
    (128256, 72, ((0.0, 2, 1, 32), (1.0, 2, 375, 24))),           # the vocabulary of the four-level configuration
])
def test_vocabulary_above_the_fused_sampler_limit(vocab, wseed, cases):
    """Hierarchies whose vocabulary (33001: above 32768, not a multiple of 4; 128256: the largest workload's) takes
    the sliced softmax and the multi-workgroup accept / resample kernel: streams against the oracle at temperature 0
    and 1.  With 1e-5 to 3e-5 of mass per token a draw's margin is bounded by the token's own width, so the asserted
    margin is 1e-6 of the mass, still ten times the fp32 differences between the two softmaxes.  Prompt and sampling
    seeds: tests/scan_stream_seeds.py."""
    shape = dict(n_layers=4, d=128, n_q=2, n_kv=2, hd=64, ffn=256, vocab=vocab)
    exits, T = (1, 2, 4), (3, 2)
    w = inputs.make_weights(shape, seed=wseed, bf16=False)
    model = gpu_model(shape, w, False, max_seq=128, max_rows=16)
    for temperature, pseed, seed, n in cases:
        prompt = inputs.make_prompt(shape["vocab"], 24, seed=pseed)
        levels = _oracle_levels(w, shape, exits, temperature, max_len=128)
        ch = specsample.PhiloxChooser(seed)
        o = ohsd.HSD(levels, T, ch)
        ref = o.generate([int(t) for t in prompt], n)
        if temperature == 0:
            assert min(l.min_top2_gap for l in levels) > 1.5e-3
        else:
            assert min(ch.accept_margins) > 3e-4 and min(ch.sample_margins) > 1e-6
        h = _gpu_hier(model, exits, T, temperature, seed=seed)
        h.prefill(prompt)
        got, st = h.generate(n)
        assert got.tolist() == ref, temperature
        assert [st.passes[i] for i in range(3)] == o.passes and [st.accepted[i] for i in range(3)] == o.accepted
        say("vocabulary", vocab, "temperature", temperature, "accepted", o.accepted, "of", o.drafted)
        h.close()
    model.close()


def test_distilled_drafters_follow_the_oracle():
    """Synthetic drafters (a foreign small network and an early exit whose logits are replaced by the target's plus
    seeded Gaussian noise of std 1.0 / 0.5): stream, pass counts and acceptance counters against the oracle, and
    the noise rows themselves."""
    from oracle import distill
    from paper_2510_19705_amd import hsd
    small = dict(n_layers=2, d=128, n_q=2, n_kv=1, hd=64, ffn=384, vocab=TINY["vocab"])
    wa = inputs.make_weights(small, seed=51, bf16=False)
    wb = inputs.make_weights(TINY, seed=1, bf16=False)
    ma = gpu_model(small, wa, False, max_seq=256, max_rows=16)
    mb = gpu_model(TINY, wb, False, max_seq=256, max_rows=16)
    da, db = oracle_decoder(small, wa, 256), oracle_decoder(TINY, wb, 256)
    prompt = inputs.make_prompt(TINY["vocab"], 32, seed=2)
    seed, T = 1301, (3, 2)
    tgt = decoder.Level(db, 8, 1.0)
    levels = [distill.DistilledLevel(da, 2, tgt, 0, 1.0, seed, 1.0), distill.DistilledLevel(db, 4, tgt, 1, 0.5, seed, 1.0), tgt]
    ch = specsample.PhiloxChooser(seed)
    o = ohsd.HSD(levels, T, ch)
    ref = o.generate([int(t) for t in prompt], 48)
    assert min(ch.accept_margins) > 3e-4 and min(ch.sample_margins) > 3e-6
    h = hsd.Hierarchy([(ma, 2), (mb, 4), (mb, 8)], T, 1.0, seed)
    h.set_distilled(0, 2, 1.0)
    h.set_distilled(1, 2, 0.5)
    h.prefill(prompt)
    got, st = h.generate(48)
    assert got.tolist() == ref
    assert [st.passes[i] for i in range(3)] == o.passes                  # the source's side passes are not counted
    assert [st.accepted[i] for i in range(3)] == o.accepted and [st.tested[i] for i in range(3)] == o.tested
    say("distilled drafters: accepted", o.accepted, "tested", o.tested)
    # the first draft row after a rewind: softmax(target logits + noise) against the oracle's row
    h.rewind(len(prompt))
    toks, q = h.draft(1)
    db.reset()
    da.reset()
    row = levels[0].next_dists([int(t) for t in prompt], 1)[0]
    assert np.abs(q.cpu().numpy()[0] - row).max() < 2e-6 * row.max() + 1e-9
    with pytest.raises(hsd.HsdError):
        h.set_distilled(2, 2, 1.0)                                       # the target is never synthetic
    with pytest.raises(hsd.HsdError):
        h.set_distilled(1, 0, 1.0)                                       # the source must be above
    h.set_distilled(0, -1, 0.0)
    h.set_distilled(1, -1, 0.0)
    h.close()
    ma.close()
    mb.close()


def test_chain_of_distilled_drafters_follows_the_oracle(tiny):
    """A chain of synthetic drafters over exits of one network (exit 2 = exit 4's logits + noise, exit 4 = the target's
    + noise): stream, pass counts and acceptance counters against the oracle, whose chained level adds the two noise
    rows to the target's logits; neighbours accept more than the single-noise configuration's ends would."""
    from oracle import distill
    from paper_2510_19705_amd import hsd
    w, prompt, model = tiny
    dec = oracle_decoder(TINY, w, 256)
    seed, T = 1403, (3, 2)
    tgt = decoder.Level(dec, 8, 1.0)
    mid = distill.DistilledLevel(dec, 4, tgt, 1, 0.5, seed, 1.0)
    low = distill.DistilledLevel(dec, 2, mid, 0, 0.5, seed, 1.0)
    ch = specsample.PhiloxChooser(seed)
    o = ohsd.HSD([low, mid, tgt], T, ch)
    ref = o.generate([int(t) for t in prompt], 48)
    say("chain: oracle margins accept %.2e sample %.2e; accepted %s of %s" % (min(ch.accept_margins), min(ch.sample_margins), o.accepted, o.drafted))
    assert min(ch.accept_margins) > 3e-4 and min(ch.sample_margins) > 3e-6
    h = hsd.Hierarchy([(model, 2), (model, 4), (model, 8)], T, 1.0, seed)
    h.set_distilled(1, 2, 0.5)
    h.set_distilled(0, 1, 0.5)
    h.prefill(prompt)
    got, st = h.generate(48)
    assert got.tolist() == ref
    assert [st.passes[i] for i in range(3)] == o.passes
    assert [st.accepted[i] for i in range(3)] == o.accepted and [st.tested[i] for i in range(3)] == o.tested
    h.close()


def test_set_seed_switches_the_sample_path(tiny):
    """hsd_hier_set_seed + rewind continue the same prompt along the sample path of another seed: equal to a
    hierarchy created with that seed, and back to the first path with the first seed."""
    w, prompt, model = tiny
    T = (3, 2)
    def fresh(seed):
        h = _gpu_hier(model, TINY_EXITS, T, 1.0, seed=seed)
        h.prefill(prompt)
        out = h.generate(40)[0].tolist()
        return h, out
    ha, a = fresh(11)
    hb, b = fresh(12)
    hb.close()
    assert a != b
    ha.set_seed(12)
    ha.rewind(len(prompt))
    assert ha.generate(40)[0].tolist() == b
    ha.set_seed(11)
    ha.rewind(len(prompt))
    assert ha.generate(40)[0].tolist() == a
    ha.close()
