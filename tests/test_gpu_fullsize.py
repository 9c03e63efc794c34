"""Full-size check of the bench workload's shape (1B-shaped bf16 model, exits 2 / 6 / 16, prompt 512) in the launch
configuration bench.py times: draft-step and verify-pass logits against the fp64 oracle, all 32000 entries per row."""
import numpy as np
import pytest

from paper_2510_19705_amd import inputs
from helpers import gpu_model, oracle_decoder, say

pytestmark = pytest.mark.gpu


def test_1b_shape_passes_match_oracle():
    import torch
    shape = inputs.SHAPES["1b"]
    say("generating 1B-shaped weights")
    w = inputs.make_weights(shape, seed=77, bf16=True)
    toks = inputs.make_prompt(shape["vocab"], 530, seed=78)
    model = gpu_model(shape, w, True, max_seq=1024, max_rows=64, rows_copy_layers=2)
    say("oracle: 16 layers over 519 tokens in fp64")
    oracle = oracle_decoder(shape, w, 640)
    ref_all = oracle.forward([int(t) for t in toks[:519]], 0, 16)          # fills the oracle cache for every layer
    td = torch.from_numpy(toks).cuda()
    for p0 in range(0, 512, 64):
        model.model_pass(td[p0:p0 + 64], p0, 16, 0)
    # verify pass of the target: 7 rows (pending token + 6 drafts)
    got = model.model_pass(td[512:519], 512, 16, 7).cpu().numpy()
    err = np.abs(got - ref_all[512:519]).max()
    say("target verify pass, 7 rows: max abs err %.3e (|z| max %.2f)" % (err, np.abs(ref_all[512:519]).max()))
    assert err < 2e-2
    # verify pass of the middle level (exit 6), 5 rows, and a one-token draft step of exit 2 (row kernel)
    ref6 = oracle.forward([int(t) for t in toks[519:524]], 519, 6)
    got6 = model.model_pass(td[519:524], 519, 6, 5).cpu().numpy()
    err6 = np.abs(got6 - ref6).max()
    say("exit-6 verify pass, 5 rows: max abs err %.3e" % err6)
    assert err6 < 2e-2
    ref2 = oracle.forward([int(toks[524])], 524, 2)
    got2 = model.model_pass(td[524:525], 524, 2, 1).cpu().numpy()
    err2 = np.abs(got2 - ref2).max()
    say("exit-2 draft step: max abs err %.3e" % err2)
    assert err2 < 2e-2
    # the distributions the sampler sees: softmax rows within 1e-3 of the oracle's in total variation
    from oracle import decoder
    from paper_2510_19705_amd import hsd
    p_gpu = hsd.softmax(torch.from_numpy(got).cuda(), 1.0).cpu().numpy().astype(np.float64)
    p_ref = decoder.distributions(ref_all[512:519], 1.0).astype(np.float64)
    tv = 0.5 * np.abs(p_gpu - p_ref).sum(axis=1).max()
    say("largest total-variation distance of a row: %.3e" % tv)
    assert tv < 5e-3
    model.close()


@pytest.mark.parametrize("name,shape,rows", [
    # one layer of the 7B shape: K = 4096 everywhere, the range where the GEMMs issue twice as many loads per batch
    ("7b_layer", dict(inputs.SHAPES["7b"], n_layers=1, vocab=8000), 6),
    # a q/k/v matrix of 138 MB in 384 column groups: the one case whose RoPE GEMM splits K over four workgroups
    ("wide_qkv_layer", dict(n_layers=1, d=5632, n_q=64, n_kv=16, hd=128, ffn=1024, vocab=1000), 6),
    # the widths of the four-level configuration, each with its 128256-row head: the 8B shape (FFN 14336, grouped heads)
    # and the 70B shape (d 8192, 64 query / 8 KV heads, FFN 28672: K >= 8192 plans, the residual projection split along K)
    ("8b_layer", dict(inputs.SHAPES["8b"], n_layers=1), 4),
    ("70b_layer", dict(inputs.SHAPES["70b"], n_layers=1), 4),
])
def test_large_layer_shapes_match_oracle(name, shape, rows):
    """Layers at the larger configurations' real widths, in the launch plans those widths select, against the fp64
    oracle: prefill of 64 tokens in one pass, then a verify pass of `rows` rows and a one-token pass; every logit of
    every row (up to 128256 per row) within 2e-2."""
    import torch
    say("generating", name)
    w = inputs.make_weights(shape, seed=91, bf16=True)
    n_tok = 64 + rows + 1
    toks = inputs.make_prompt(shape["vocab"], n_tok, seed=92)
    model = gpu_model(shape, w, True, max_seq=128, max_rows=64)
    say("  oracle:", name)
    oracle = oracle_decoder(shape, w, 128)
    ref = oracle.forward([int(t) for t in toks], 0, 1)
    del oracle
    td = torch.from_numpy(toks).cuda()
    got64 = model.model_pass(td[:64], 0, 1, 64).cpu().numpy()
    gotr = model.model_pass(td[64:64 + rows], 64, 1, rows).cpu().numpy()
    got1 = model.model_pass(td[64 + rows:], 64 + rows, 1, 1).cpu().numpy()
    for tag, got, want in (("64-row pass", got64, ref[:64]), ("%d-row pass" % rows, gotr, ref[64:64 + rows]),
                           ("1-row pass", got1, ref[64 + rows:])):
        err = np.abs(got - want).max()
        say("  %s %s: max abs err %.3e (|z| max %.2f)" % (name, tag, err, np.abs(want).max()))
        assert err < 2e-2, (name, tag)
    model.close()
