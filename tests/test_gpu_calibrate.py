"""GPU parity of the calibration pass (Sec. 5.1): several exits in one pass, the overlap kernel, the all-pairs
acceptance matrix and the selection it feeds, against the fp64 oracle."""
import numpy as np
import pytest

from oracle import calibrate, latency
from paper_2510_19705_amd import inputs
from helpers import gpu_model, oracle_decoder, say

pytestmark = pytest.mark.gpu

SMALL_F32 = dict(n_layers=4, d=96, n_q=6, n_kv=2, hd=32, ffn=160, vocab=777)
SMALL_BF16 = dict(n_layers=6, d=256, n_q=8, n_kv=2, hd=64, ffn=608, vocab=5000)


def _cuda(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
def test_pass_exits_equals_single_exit_passes(bf16):
    """Every exit's logits from the one multi-exit pass are bit-identical to that exit's own pass, and within the
    storage type's tolerance of the oracle; the pass also leaves the same K/V behind (a later pass agrees)."""
    import torch
    shape = SMALL_BF16 if bf16 else SMALL_F32
    w = inputs.make_weights(shape, seed=31, bf16=bf16)
    toks = inputs.make_prompt(shape["vocab"], 90, seed=32)
    L = shape["n_layers"]
    exits = [1, 2, L - 1, L] if bf16 else [1, 3, L]
    a = gpu_model(shape, w, bf16, max_seq=128, max_rows=24)
    b = gpu_model(shape, w, bf16, max_seq=128, max_rows=24)
    oracle = oracle_decoder(shape, w, 128)
    td = _cuda(toks.astype(np.int32))
    for (pos0, m, nl) in [(0, 24, 0), (24, 24, 5), (48, 7, 7), (55, 1, 1), (56, 20, 20)]:
        multi = a.model_pass_exits(td[pos0:pos0 + m], pos0, exits, nl)
        oracle.forward([int(t) for t in toks[pos0:pos0 + m]], pos0, L)          # fills every layer's oracle cache
        for i, e in enumerate(exits):
            single = b.model_pass(td[pos0:pos0 + m], pos0, e, nl)
            if nl:
                assert torch.equal(multi[i], single), (pos0, m, e)
                ref = oracle.forward([int(t) for t in toks[pos0:pos0 + m]], pos0, e)[m - nl:]
                err = np.abs(multi[i].cpu().numpy() - ref).max()
                assert err < (2e-2 if bf16 else 1e-4 * np.abs(ref).max()), (pos0, m, e, err)
    # the caches of the two models agree: one more deep pass gives identical logits
    x = a.model_pass(td[76:80], 76, L, 4)
    y = b.model_pass(td[76:80], 76, L, 4)
    assert torch.equal(x, y)
    from paper_2510_19705_amd import hsd
    with pytest.raises(hsd.HsdError) as e:
        a.model_pass_exits(td[:4], 0, [2, 2], 1)             # not ascending
    assert e.value.code == -1
    with pytest.raises(hsd.HsdError):
        a.model_pass_exits(td[:4], 0, [1, L + 1], 1)
    a.close()
    b.close()


@pytest.mark.parametrize("n,R,V", [(2, 1, 50), (3, 7, 2048), (5, 16, 5001), (4, 3, 32000)])
def test_overlap_kernel(n, R, V):
    from paper_2510_19705_amd import hsd
    rng = np.random.default_rng(n * 100 + R)
    z = rng.standard_normal((n, R, V)) * 2.5
    e = np.exp(z - z.max(axis=-1, keepdims=True))
    rows = (e / e.sum(axis=-1, keepdims=True)).astype(np.float32)
    rows[0, 0, :] = 0
    rows[0, 0, 3] = 1.0                                        # a one-hot row
    got = hsd.overlap(_cuda(rows)).cpu().numpy()
    pair = 0
    for i in range(n):
        for j in range(i + 1, n):
            for r in range(R):
                assert abs(got[pair, r] - calibrate.overlap(rows[i, r], rows[j, r])) < 1e-12, (i, j, r)
            pair += 1
    assert pair == got.shape[0]


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
def test_calibrate_matrix_and_selection(bf16):
    """alpha from the library against the oracle's (fp32 storage: 1e-5; bf16: the rows differ by the logits' 2e-2, so
    5e-3 on the means), symmetric, unit diagonal, triangle inequality; the selection on the library's alpha and on
    the oracle's alpha agree when costs are fixed numbers."""
    from paper_2510_19705_amd import hsd
    shape = SMALL_BF16 if bf16 else SMALL_F32
    w = inputs.make_weights(shape, seed=41, bf16=bf16)
    L = shape["n_layers"]
    exits = [1, 2, 4, L] if bf16 else [1, 2, L]
    toks = inputs.make_prompt(shape["vocab"], 75, seed=42)
    model = gpu_model(shape, w, bf16, max_seq=128, max_rows=24)
    alpha, cost = model.calibrate(exits, _cuda(toks.astype(np.int32)), 30, 1.0, cost_rows=4)
    rows = calibrate.exit_distributions(oracle_decoder(shape, w, 128), exits, toks, 30, 1.0)
    ref = calibrate.acceptance_matrix(rows)
    say("alpha library\n", np.round(alpha, 4), "\nalpha oracle\n", np.round(ref, 4), "\ncost ms", cost)
    assert np.abs(alpha - ref).max() < (5e-3 if bf16 else 1e-5)
    assert np.array_equal(alpha, alpha.T) and (np.diag(alpha) == 1).all()
    assert calibrate.triangle_violation(alpha) <= 1e-9
    assert (cost > 0).all() and cost[-1] > cost[0]            # deeper exits cost more
    # no context-only positions, fewer positions than one chunk
    a_short, _ = model.calibrate(exits, _cuda(toks[:11].astype(np.int32)), 0, 1.0)
    r_short = calibrate.acceptance_matrix(calibrate.exit_distributions(oracle_decoder(shape, w, 128), exits, toks[:11], 0, 1.0))
    assert np.abs(a_short - r_short).max() < (8e-3 if bf16 else 1e-5)
    # temperature 0: one-hot rows, overlap = fraction of positions where the argmaxes agree
    a0, _ = model.calibrate(exits, _cuda(toks.astype(np.int32)), 30, 0.0)
    r0 = calibrate.acceptance_matrix(calibrate.exit_distributions(oracle_decoder(shape, w, 128), exits, toks, 30, 0.0))
    if not bf16:
        assert np.array_equal(a0, r0)
    assert set(np.unique(np.round(a0 * 45).astype(int))).issubset(set(range(46)))
    # selection (Sec. 4) on measured alpha with synthetic costs proportional to depth + head
    n = len(exits)
    c = [e + 1.5 for e in exits]
    got = hsd.select_hierarchy(c, alpha, 6)
    want = latency.select_hierarchy(c, ref, 6)
    say("selected", got, "oracle", want)
    assert abs(got[0] - want[0]) < (2e-2 if bf16 else 1e-4) * want[0]
    if not bf16:
        assert list(got[1]) == list(want[1]) and list(got[2]) == list(want[2])
    # bad arguments
    with pytest.raises(hsd.HsdError):
        model.calibrate(exits, _cuda(toks.astype(np.int32)), 75, 1.0)       # nothing to score
    with pytest.raises(hsd.HsdError):
        model.calibrate([2, 1], _cuda(toks.astype(np.int32)), 30, 1.0)
    model.close()


def test_calibrate_levels_across_networks():
    """Candidates from two networks (a small independent drafter; three exits of a second network, listed between and
    after it) in one call: the acceptance matrix against the oracle's rows of each candidate, indexed by candidate
    whatever the order the networks are scored in; costs positive; every network's cache left filled (a later pass of
    each agrees with a freshly prefilled copy); bad candidate lists are refused."""
    import torch
    from paper_2510_19705_amd import hsd
    big = SMALL_F32
    small = dict(n_layers=2, d=64, n_q=2, n_kv=1, hd=32, ffn=96, vocab=big["vocab"])
    wb, ws = inputs.make_weights(big, seed=43, bf16=False), inputs.make_weights(small, seed=44, bf16=False)
    toks = inputs.make_prompt(big["vocab"], 70, seed=45)
    mb, ms = gpu_model(big, wb, False, max_seq=128, max_rows=24), gpu_model(small, ws, False, max_seq=128, max_rows=8)
    cands = [(mb, 1), (ms, 2), (mb, 3), (mb, 4)]
    td = _cuda(toks.astype(np.int32))
    alpha, cost = hsd.calibrate_levels(cands, td, 25, 1.0, cost_rows=4)
    rows_b = calibrate.exit_distributions(oracle_decoder(big, wb, 128), [1, 3, 4], toks, 25, 1.0)
    rows_s = calibrate.exit_distributions(oracle_decoder(small, ws, 128), [2], toks, 25, 1.0)
    ref = calibrate.acceptance_matrix(np.stack([rows_b[0], rows_s[0], rows_b[1], rows_b[2]]))
    say("alpha library\n", np.round(alpha, 4), "\nalpha oracle\n", np.round(ref, 4), "\ncost ms", cost)
    assert np.abs(alpha - ref).max() < 1e-5
    assert np.array_equal(alpha, alpha.T) and (np.diag(alpha) == 1).all() and (cost > 0).all()
    assert calibrate.triangle_violation(alpha) <= 1e-9
    # the call doubles as a prefill: one more pass of each network equals the same pass after a plain prefill
    for model, shape, w, e in ((mb, big, wb, 4), (ms, small, ws, 2)):
        fresh = gpu_model(shape, w, False, max_seq=128, max_rows=24)
        for p0 in range(0, 66, 22):
            fresh.model_pass(td[p0:p0 + 22], p0, e, 0)
        assert torch.equal(model.model_pass(td[66:70], 66, e, 4), fresh.model_pass(td[66:70], 66, e, 4))
        fresh.close()
    with pytest.raises(hsd.HsdError):
        hsd.calibrate_levels([(mb, 3), (ms, 2), (mb, 1)], td, 25, 1.0)          # exits of one network out of order
    other = gpu_model(dict(small, vocab=500), inputs.make_weights(dict(small, vocab=500), seed=46, bf16=False), False, 128, 8)
    with pytest.raises(hsd.HsdError):
        hsd.calibrate_levels([(other, 1), (mb, 4)], td, 25, 1.0)                # different vocabularies
    for m in (mb, ms, other):
        m.close()
