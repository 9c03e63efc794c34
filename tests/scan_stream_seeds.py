#!/usr/bin/env python3
"""Regenerates the prompt / sampling seeds that the GPU stream tests use.  CPU only, oracle only.

A stream test compares the library's token stream with the oracle's token by token, which is only well-posed when
every decision of the oracle's run keeps a margin far above the rounding differences between the two sides: at
temperature 0 the gap between the two largest logits of every row, at temperature 1 the distance of every accept
test from its threshold and of every draw from the ends of its token's interval.  The tests assert those margins;
this script is how the values they use were found and how they can be found again after a change of the oracle:

    python tests/scan_stream_seeds.py                  # check the values in use (prints the margins of each case)
    python tests/scan_stream_seeds.py --search         # for every case: the first value of the scanned range that qualifies
    python tests/scan_stream_seeds.py --search --case vocab_128256_t1
    python tests/scan_stream_seeds.py --batch          # the (prompt, length, seed) triples of tests/test_gpu_batch.py

The two tests with synthetic drafters (test_distilled_drafters_follow_the_oracle, seed 1301, and
test_chain_of_distilled_drafters_follows_the_oracle, seed 1403) draw noise from the same seed as the sampler, so their
seed is found by running the test's own oracle block over consecutive seeds from 1300 / 1400 and taking the first
one whose margins pass the test's assertion.

At temperature 0 the sampling seed is irrelevant and the PROMPT seed is scanned; at temperature 1 the prompt is kept
and the SAMPLING seed is scanned.  Nothing here touches the GPU or the library.
"""
import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

from oracle import decoder, distill, hsd as ohsd, specsample      # noqa: E402
from paper_2510_19705_amd import inputs                           # noqa: E402
from helpers import oracle_decoder                                # noqa: E402

TINY = inputs.SHAPES["tiny"]
SMALL = dict(n_layers=2, d=128, n_q=2, n_kv=1, hd=64, ffn=384, vocab=TINY["vocab"])
V33K = dict(n_layers=4, d=128, n_q=2, n_kv=2, hd=64, ffn=256, vocab=33001)
V128K = dict(n_layers=4, d=128, n_q=2, n_kv=2, hd=64, ffn=256, vocab=128256)

# name: networks [(shape, weight seed)], levels [(network index, exit)], T, temperature, prompt length, tokens,
# margins (top-2 gap | accept, sample), the value in use (prompt seed at temperature 0, else (prompt seed, sampling seed)),
# and the test that uses it
CASES = {
    "tiny_t0": dict(nets=[(TINY, 1)], levels=[(0, 2), (0, 4), (0, 8)], T=[(4, 2), (2, 4)], temp=0.0, n_prompt=32, n=64,
                    gap=1.5e-3, use=10, test="test_tiny_temperature0_stream_bit_exact, test_temperature0_random_hierarchies"),
    "tiny_t1_T4_2": dict(nets=[(TINY, 1)], levels=[(0, 2), (0, 4), (0, 8)], T=[(4, 2)], temp=1.0, n_prompt=32, n=64,
                         acc=3e-4, samp=3e-6, use=(2, 104), test="test_tiny_temperature1_stream"),
    "tiny_t1_T3_5": dict(nets=[(TINY, 1)], levels=[(0, 2), (0, 4), (0, 8)], T=[(3, 5)], temp=1.0, n_prompt=32, n=64,
                         acc=3e-4, samp=3e-6, use=(2, 100), test="test_tiny_temperature1_stream"),
    "independent_t0": dict(nets=[(SMALL, 51), (TINY, 1)], levels=[(0, 2), (1, 4), (1, 8)], T=[(3, 2)], temp=0.0, n_prompt=32, n=48,
                           gap=1.5e-3, use=73, test="test_independent_models_in_one_hierarchy"),
    "independent_t1": dict(nets=[(SMALL, 51), (TINY, 1)], levels=[(0, 2), (1, 4), (1, 8)], T=[(3, 2)], temp=1.0, n_prompt=32, n=48,
                           acc=3e-4, samp=3e-6, use=(2, 305), test="test_independent_models_in_one_hierarchy"),
    "eight_levels_t0": dict(nets=[(TINY, 1)], levels=[(0, e) for e in range(1, 9)], T=[(2, 1, 1, 1, 1, 1, 1)], temp=0.0, n_prompt=32,
                            n=40, gap=1e-3, use=11, test="test_largest_hierarchies"),
    "eight_levels_t1": dict(nets=[(TINY, 1)], levels=[(0, e) for e in range(1, 9)], T=[(2, 1, 1, 1, 1, 1, 1)], temp=1.0, n_prompt=32,
                            n=40, acc=3e-4, samp=3e-6, use=(2, 801), test="test_largest_hierarchies"),
    "forty_drafts_t0": dict(nets=[(TINY, 1)], levels=[(0, 2), (0, 8)], T=[(40,)], temp=0.0, n_prompt=32, n=90, gap=1e-3, use=12,
                            test="test_largest_hierarchies"),
    "forty_drafts_t1": dict(nets=[(TINY, 1)], levels=[(0, 2), (0, 8)], T=[(40,)], temp=1.0, n_prompt=32, n=90, acc=3e-4, samp=3e-6,
                            use=(2, 811), test="test_largest_hierarchies"),
    "vocab_33001_t0": dict(nets=[(V33K, 71)], levels=[(0, 1), (0, 2), (0, 4)], T=[(3, 2)], temp=0.0, n_prompt=24, n=32, gap=1.5e-3,
                           use=30, test="test_vocabulary_above_the_fused_sampler_limit"),
    "vocab_33001_t1": dict(nets=[(V33K, 71)], levels=[(0, 1), (0, 2), (0, 4)], T=[(3, 2)], temp=1.0, n_prompt=24, n=24, acc=3e-4,
                           samp=1e-6, use=(2, 911), test="test_vocabulary_above_the_fused_sampler_limit"),
    "vocab_128256_t0": dict(nets=[(V128K, 72)], levels=[(0, 1), (0, 2), (0, 4)], T=[(3, 2)], temp=0.0, n_prompt=24, n=32, gap=1.5e-3,
                            use=2, test="test_vocabulary_above_the_fused_sampler_limit"),
    "vocab_128256_t1": dict(nets=[(V128K, 72)], levels=[(0, 1), (0, 2), (0, 4)], T=[(3, 2)], temp=1.0, n_prompt=24, n=24, acc=3e-4,
                            samp=1e-6, use=(2, 375), test="test_vocabulary_above_the_fused_sampler_limit"),
}


def margins(case, decoders, pseed, seed):
    """Runs the oracle for every T of the case; returns (worst top-2 gap, worst accept margin, worst sample margin)."""
    vocab = case["nets"][0][0]["vocab"]
    prompt = [int(t) for t in inputs.make_prompt(vocab, case["n_prompt"], seed=pseed)]
    gap, acc, samp = float("inf"), float("inf"), float("inf")
    for T in case["T"]:
        for d in decoders:
            d.reset()
        levels = [decoder.Level(decoders[i], e, case["temp"]) for i, e in case["levels"]]
        ch = specsample.PhiloxChooser(seed)
        ohsd.HSD(levels, T, ch).generate(prompt, case["n"])
        gap = min(gap, min(l.min_top2_gap for l in levels))
        acc = min([acc] + ch.accept_margins)
        samp = min([samp] + ch.sample_margins)
    return gap, acc, samp


def qualifies(case, m):
    if case["temp"] == 0:
        return m[0] > case["gap"]
    return m[1] > case["acc"] and m[2] > case["samp"]


def batch_sequences():
    """The (prompt seed, prompt length, sampling seed) triples of tests/test_gpu_batch.py: 48 tokens, T = (4, 2), prompt
    lengths 24 / 32 / 40 by prompt seed; temperature 1: for prompt seeds 2..7 the first sampling seed from
    200 + 10 * prompt seed on that qualifies; temperature 0: the prompt seeds from 10 on whose greedy run qualifies."""
    case = dict(CASES["tiny_t1_T4_2"], n=48)
    decoders = [oracle_decoder(shape, inputs.make_weights(shape, seed=ws, bf16=False), 40 + 48 + 64) for shape, ws in case["nets"]]
    for pseed in range(2, 8):
        case["n_prompt"] = 24 + (pseed % 3) * 8
        for v in range(60):
            m = margins(case, decoders, pseed, 200 + 10 * pseed + v)
            if qualifies(case, m):
                print("temperature 1: (%d, %d, %d)  accept %.2e sample %.2e" % (pseed, case["n_prompt"], 200 + 10 * pseed + v, m[1], m[2]), flush=True)
                break
    case0 = dict(CASES["tiny_t0"], T=[(4, 2)], n=48)
    for pseed in range(10, 30):
        case0["n_prompt"] = 24 + (pseed % 3) * 8
        m = margins(case0, decoders, pseed, 1)
        if qualifies(case0, m):
            print("temperature 0: (%d, %d, 1)  top-2 gap %.2e" % (pseed, case0["n_prompt"], m[0]), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--search", action="store_true", help="scan for the first qualifying value instead of checking the one in use")
    ap.add_argument("--case", action="append", help="only these cases (default: all)")
    ap.add_argument("--limit", type=int, default=400, help="values scanned per case")
    ap.add_argument("--batch", action="store_true", help="the sequences of tests/test_gpu_batch.py")
    args = ap.parse_args()
    if args.batch:
        batch_sequences()
        return
    for name, case in CASES.items():
        if args.case and name not in args.case:
            continue
        max_len = case["n_prompt"] + case["n"] + 64
        decoders = [oracle_decoder(shape, inputs.make_weights(shape, seed=ws, bf16=False), max_len) for shape, ws in case["nets"]]
        if not args.search:
            if case["use"] is None:
                print("%s: no value in use yet" % name, flush=True)
                continue
            pseed, seed = (case["use"], 1) if case["temp"] == 0 else case["use"]
            m = margins(case, decoders, pseed, seed)
            print("%s (%s): prompt seed %d, sampling seed %d: top-2 gap %.2e, accept margin %.2e, sample margin %.2e -> %s"
                  % (name, case["test"], pseed, seed, m[0], m[1], m[2], "ok" if qualifies(case, m) else "DOES NOT QUALIFY"), flush=True)
            continue
        found = None
        for v in range(args.limit):
            pseed, seed = (v, 1) if case["temp"] == 0 else (2, 100 + v)
            m = margins(case, decoders, pseed, seed)
            if qualifies(case, m):
                found = (pseed, seed, m)
                break
        if found:
            print("%s: prompt seed %d, sampling seed %d qualifies (gap %.2e, accept %.2e, sample %.2e)"
                  % (name, found[0], found[1], found[2][0], found[2][1], found[2][2]), flush=True)
        else:
            print("%s: nothing in the first %d values qualifies" % (name, args.limit), flush=True)


if __name__ == "__main__":
    main()
