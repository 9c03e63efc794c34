"""GPU parity of the stand-alone kernels against the oracle (element by element, same seeded inputs)."""
import numpy as np
import pytest

from oracle import decoder, specsample
from paper_2510_19705_amd import inputs
from helpers import say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hsd():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2510_19705_amd import hsd as lib
    return lib


def _cuda(a, dtype=None):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


# ---- softmax ---------------------------------------------------------------------------------
@pytest.mark.parametrize("rows,V", [(1, 50), (3, 2048), (5, 5000), (2, 32769), (3, 40961), (17, 128256)])
@pytest.mark.parametrize("temperature", [1.0, 0.7, 0.0])
def test_softmax(hsd, rows, V, temperature):
    say("softmax", rows, V, temperature)
    rng = np.random.default_rng(rows * 7 + V)
    z = (rng.standard_normal((rows, V)) * 3).astype(np.float32)
    if rows > 1:
        z[1, 7] = z[1, V - 3] = z[1].max() + 1.0           # tie: lowest index must win
    got = hsd.softmax(_cuda(z), temperature).cpu().numpy()
    ref = decoder.distributions(z.astype(np.float64), temperature)
    if temperature == 0:
        assert (got == ref).all()
    else:
        # fp32 exp and a 1024-way fp32 sum: relative error ~1e-6 per element
        assert np.abs(got - ref).max() <= 2e-6 * ref.max() + 1e-9
        assert np.abs(got.astype(np.float64).sum(axis=1) - 1).max() < 1e-5


# ---- accept / reject / resample: bit-exact on the oracle's probabilities and Philox stream ------
@pytest.mark.parametrize("V", [50, 2048, 5000, 128256])
@pytest.mark.parametrize("t", [0, 1, 4, 16])
def test_accept_resample_bit_exact(hsd, V, t):
    import torch
    say("accept_resample", V, t)
    seed = 0x1234ABCD5678EF01
    n_calls = 40 if V < 100000 else 12
    n_hist = np.zeros(t + 2, dtype=int)
    for call in range(n_calls):
        p, q, x = inputs.make_prob_rows(V, t, seed=1000 * V + 17 * t + call, sigma=2.0 + (call % 3), noise=0.3 + 0.5 * (call % 4))
        ch = specsample.PhiloxChooser(seed)
        n_ref, m_ref = specsample.verify(list(p), list(q), list(x), ch, level=3, call=call)
        xd = _cuda(np.concatenate([x, [0]]).astype(np.int32))
        n, m = hsd.accept_resample(_cuda(p), _cuda(q) if t else _cuda(p[:0]), xd, seed, 3, call)
        assert (n, m) == (n_ref, m_ref), (V, t, call)
        assert int(xd[n].item()) == m_ref
        n_hist[n] += 1
    say("  accepted-count histogram", n_hist.tolist())
    if t >= 4:
        assert (n_hist > 0).sum() >= 2                     # both rejections and acceptances were exercised


@pytest.mark.parametrize("V", [32000, 32768, 32769, 40000])
def test_accept_resample_kernel_boundary(hsd, V):
    """Vocabularies around the switch between the one-workgroup and the multi-workgroup kernel."""
    seed = 99
    for call in range(10):
        p, q, x = inputs.make_prob_rows(V, 5, seed=V + call, sigma=3.0, noise=0.6)
        ref = specsample.verify(list(p), list(q), list(x), specsample.PhiloxChooser(seed), 2, call)
        xd = _cuda(np.concatenate([x, [0]]).astype(np.int32))
        assert hsd.accept_resample(_cuda(p), _cuda(q), xd, seed, 2, call) == ref, (V, call)


def test_accept_resample_degenerate_rows(hsd):
    import torch
    V, seed = 3000, 77
    # one-hot rows (temperature 0): accept iff the draft equals the verifier's argmax
    p, q, x = inputs.make_prob_rows(V, 3, seed=5, one_hot=True)
    q[0] = p[0]
    x[0] = int(np.argmax(p[0]))                            # first draft agrees, second may not
    for call in range(6):
        ref = specsample.verify(list(p), list(q), list(x), specsample.PhiloxChooser(seed), 1, call)
        xd = _cuda(np.concatenate([x, [0]]).astype(np.int32))
        assert hsd.accept_resample(_cuda(p), _cuda(q), xd, seed, 1, call) == ref
        assert ref[0] >= 1
    # p == q exactly: every draft is accepted unless u*q rounds up to p; the residual is identically zero
    p, q, x = inputs.make_prob_rows(V, 4, seed=6)
    q = p[:4].copy()
    for call in range(6):
        ref = specsample.verify(list(p), list(q), list(x), specsample.PhiloxChooser(seed), 2, call)
        xd = _cuda(np.concatenate([x, [0]]).astype(np.int32))
        assert hsd.accept_resample(_cuda(p), _cuda(q), xd, seed, 2, call) == ref
    # a draft the verifier gives zero mass is always rejected and never resampled
    p, q, x = inputs.make_prob_rows(V, 2, seed=8)
    p[0, x[0]] = 0.0
    ref = specsample.verify(list(p), list(q), list(x), specsample.PhiloxChooser(seed), 1, 0)
    xd = _cuda(np.concatenate([x, [0]]).astype(np.int32))
    got = hsd.accept_resample(_cuda(p), _cuda(q), xd, seed, 1, 0)
    assert got == ref and got[0] == 0 and got[1] != x[0]


# ---- softmax + Verify in one launch ----------------------------------------------------------------
@pytest.mark.parametrize("V", [50, 2050, 5000, 32000, 32768])
@pytest.mark.parametrize("t", [0, 1, 5, 16])
@pytest.mark.parametrize("temperature", [1.0, 0.6])
def test_softmax_verify_fused(hsd, V, t, temperature):
    """The fused launch against the oracle (softmax in fp64 rounded to fp32, then Alg. 2 on the Philox stream):
    equal (n, m) whenever the oracle's decisions keep a margin above the fp32 softmax error (nearly always;
    counted), probabilities to fp32 accuracy; and bit-identical to the two stand-alone launches always."""
    import torch
    say("softmax_verify", V, t, temperature)
    seed = 0xC0FFEE1234
    checked = 0
    n_calls = 16
    n_hist = np.zeros(t + 2, dtype=int)
    for call in range(n_calls):
        z, q, x = inputs.make_logit_rows(V, t, seed=77 * V + 13 * t + call, sigma=2.0 + (call % 3), noise=0.3 + 0.4 * (call % 4))
        p_ref = decoder.distributions(z.astype(np.float64), temperature).astype(np.float32)
        ch = specsample.PhiloxChooser(seed)
        n_ref, m_ref = specsample.verify(list(p_ref), list(q), list(x), ch, level=2, call=call)
        zd, qd = _cuda(z), _cuda(q) if t else _cuda(z[:0])
        xd = _cuda(np.concatenate([x, [0]]).astype(np.int32))
        mailbox = torch.zeros(t + 3, dtype=torch.int32).pin_memory()
        n, m, probs = hsd.softmax_verify(zd, qd, xd, temperature, seed, 2, call, mailbox=mailbox)
        got_p = probs.cpu().numpy()
        assert np.abs(got_p - p_ref).max() <= 2e-6 * p_ref.max() + 1e-9
        robust = min(ch.accept_margins + [1.0]) > 1e-4 and min(ch.sample_margins + [1.0]) > 3e-6
        if robust:
            checked += 1
            assert (n, m) == (n_ref, m_ref), (V, t, call)
            n_hist[n] += 1
        # the two stand-alone launches on the same inputs: identical bits
        p2 = hsd.softmax(zd, temperature)
        assert torch.equal(p2, probs)
        xd2 = _cuda(np.concatenate([x, [0]]).astype(np.int32))
        assert hsd.accept_resample(p2, qd, xd2, seed, 2, call) == (n, m)
        assert torch.equal(xd, xd2)
        assert mailbox[:2].tolist() == [n, m]
        assert mailbox[2:3 + n].tolist() == list(x[:n]) + [m]
        # without the probability rows the decision is the same
        xd3 = _cuda(np.concatenate([x, [0]]).astype(np.int32))
        assert hsd.softmax_verify(zd, qd, xd3, temperature, seed, 2, call, want_probs=False)[:2] == (n, m)
    say("  checked against the oracle:", checked, "of", n_calls, "accepted-count histogram", n_hist.tolist())
    assert checked >= n_calls - 3


@pytest.mark.parametrize("V,t", [(1, 0), (1, 3), (2, 5), (7, 64), (4097, 64), (32768, 64)])
def test_sampler_extreme_shapes(hsd, V, t):
    """The largest draft count (64), the smallest vocabularies (1 and 2 tokens: every draw is forced or a coin), and
    chunk-boundary vocabularies, through both the two-launch and the fused entry points, bit-exact on the oracle."""
    import torch
    seed = 4242
    for call in range(4):
        p, q, x = inputs.make_prob_rows(V, t, seed=9 * V + t + call, sigma=1.5, noise=0.7)
        ref = specsample.verify(list(p), list(q), list(x), specsample.PhiloxChooser(seed), 1, call)
        xd = _cuda(np.concatenate([x, [0]]).astype(np.int32))
        assert hsd.accept_resample(_cuda(p), _cuda(q) if t else _cuda(p[:0]), xd, seed, 1, call) == ref, (V, t, call)
        if V == 1:
            assert ref == (t, 0)                              # one token: always accepted, always emitted
        # fused: logits whose softmax is exactly representable are hard to come by, so compare with its own two-launch twin
        z, q2, x2 = inputs.make_logit_rows(V, t, seed=5 * V + t + call)
        zd, qd = _cuda(z), _cuda(q2) if t else _cuda(z[:0])
        xa = _cuda(np.concatenate([x2, [0]]).astype(np.int32))
        xb = xa.clone()
        n, m, probs = hsd.softmax_verify(zd, qd, xa, 1.0, seed, 1, call)
        assert hsd.accept_resample(hsd.softmax(zd, 1.0), qd, xb, seed, 1, call) == (n, m)
        assert torch.equal(xa, xb)
        p_ref = decoder.distributions(z.astype(np.float64), 1.0).astype(np.float32)
        ch = specsample.PhiloxChooser(seed)
        ref2 = specsample.verify(list(p_ref), list(q2), list(x2), ch, 1, call)
        if min(ch.accept_margins + [1.0]) > 1e-4 and min(ch.sample_margins + [1.0]) > 3e-6:
            assert (n, m) == ref2, (V, t, call)


def test_softmax_verify_greedy_and_limits(hsd):
    """Temperature 0: one-hot rows, drafts accepted iff they equal the verifier's argmax; vocabularies beyond the
    one-workgroup limit and bad arguments are refused."""
    import torch
    V, t = 4000, 4
    z, q, x = inputs.make_logit_rows(V, t, seed=3)
    q = np.zeros_like(q)
    arg = z.argmax(axis=1)
    x = arg[:t].astype(np.int32).copy()
    x[2] = (x[2] + 1) % V                                    # third draft disagrees
    q[np.arange(t), x] = 1.0
    xd = _cuda(np.concatenate([x, [0]]).astype(np.int32))
    n, m, probs = hsd.softmax_verify(_cuda(z), _cuda(q), xd, 0.0, 5, 1, 0)
    p_ref = decoder.distributions(z.astype(np.float64), 0.0).astype(np.float32)
    assert (probs.cpu().numpy() == p_ref).all()
    ref = specsample.verify(list(p_ref), list(q), list(x), specsample.PhiloxChooser(5), 1, 0)
    assert (n, m) == ref == (2, int(arg[2]))
    f = hsd.lib.hsd_softmax_verify
    zz = torch.zeros((2, 40000), device="cuda")
    xx = torch.zeros(70, dtype=torch.int32, device="cuda")
    assert f(zz.data_ptr(), zz.data_ptr(), xx.data_ptr(), 1, 40000, 1.0, 0, 0, 0, None, xx.data_ptr(), xx.data_ptr(), None, None) == -2
    assert f(zz.data_ptr(), None, xx.data_ptr(), 1, 8, 1.0, 0, 0, 0, None, xx.data_ptr(), xx.data_ptr(), None, None) == -1
    assert f(zz.data_ptr(), zz.data_ptr(), xx.data_ptr(), 65, 8, 1.0, 0, 0, 0, None, xx.data_ptr(), xx.data_ptr(), None, None) == -1
    assert f(zz.data_ptr(), zz.data_ptr(), xx.data_ptr(), 1, 8, -1.0, 0, 0, 0, None, xx.data_ptr(), xx.data_ptr(), None, None) == -1


def test_accept_resample_rejects_bad_arguments(hsd):
    import torch
    p = torch.zeros((2, 8), device="cuda")
    x = torch.zeros(70, dtype=torch.int32, device="cuda")
    f = hsd.lib.hsd_accept_resample
    assert f(p.data_ptr(), None, x.data_ptr(), 1, 8, 0, 0, 0, x.data_ptr(), x.data_ptr(), None) == -1      # drafts without q rows
    assert b"draft rows" in hsd.lib.hsd_last_error()
    assert f(p.data_ptr(), p.data_ptr(), x.data_ptr(), 65, 8, 0, 0, 0, x.data_ptr(), x.data_ptr(), None) == -1
    assert f(None, p.data_ptr(), x.data_ptr(), 1, 8, 0, 0, 0, x.data_ptr(), x.data_ptr(), None) == -1
    assert f(p.data_ptr(), p.data_ptr(), x.data_ptr(), 1, 0, 0, 0, 0, x.data_ptr(), x.data_ptr(), None) == -1


# ---- small-M GEMM ----------------------------------------------------------------------------
@pytest.mark.parametrize("m,n,k", [(1, 48, 64), (5, 5000, 256), (16, 3072, 2048), (17, 2048, 8192), (33, 1000, 512),
                                   (64, 4096, 1024), (6, 32000, 2048)])
@pytest.mark.parametrize("bf16,layout", [(True, 0), (True, 1), (False, 0)], ids=["bf16_tiles", "bf16_rows", "f32"])
def test_gemm(hsd, m, n, k, bf16, layout):
    import torch
    say("gemm", m, n, k, "bf16" if bf16 else "f32", "layout", layout)
    rng = np.random.default_rng(m * 1000 + n + k)
    x = rng.standard_normal((m, k)).astype(np.float32)
    w = (rng.standard_normal((n, k)) / np.sqrt(k)).astype(np.float32)
    if bf16:
        x, w = inputs.bf16_round(x), inputs.bf16_round(w)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    dt = hsd.BF16 if bf16 else hsd.F32
    td = torch.bfloat16 if bf16 else torch.float32
    packed = hsd.pack_weight(_cuda(w, td), dt, layout)
    got = hsd.gemm(_cuda(x, td), packed, n, dt, None, layout).cpu().numpy()
    # exact products, fp32 accumulation over k terms in a few partial sums
    tol = 4e-6 * np.sqrt(k) * np.abs(ref).max() + 1e-6
    assert np.abs(got - ref).max() < tol, (np.abs(got - ref).max(), tol)


@pytest.mark.parametrize("m,n,k", [(65, 1000, 512), (128, 4096, 1024), (200, 520, 96), (513, 300, 2048), (1024, 2048, 4096),
                                   (1000, 48, 32)])
@pytest.mark.parametrize("path", ["tiled_for_mfma", "stream_per_64_rows"])
def test_gemm_many_rows(hsd, m, n, k, path):
    """More than 64 rows (a batch of sequences times their drafted tokens): the kernel tiled for the matrix cores
    (ragged row / column blocks, an odd number of 32-wide k tiles, fewer columns than one workgroup's strip) and the
    one-stream-per-64-rows path against the fp64 product of the same bf16 inputs."""
    import torch
    say("gemm_many_rows", m, n, k, path)
    rng = np.random.default_rng(m * 7 + n + k)
    x = inputs.bf16_round(rng.standard_normal((m, k)).astype(np.float32))
    w = inputs.bf16_round((rng.standard_normal((n, k)) / np.sqrt(k)).astype(np.float32))
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    packed = hsd.pack_weight(_cuda(w, torch.bfloat16), hsd.BF16, 0)
    tuning = hsd.kernel_tuning(wide_min_rows=65 if path == "tiled_for_mfma" else 1 << 30)
    got = hsd.gemm(_cuda(x, torch.bfloat16), packed, n, hsd.BF16, None, 0, tuning).cpu().numpy()
    tol = 4e-6 * np.sqrt(k) * np.abs(ref).max() + 1e-6
    assert np.abs(got - ref).max() < tol, (np.abs(got - ref).max(), tol)


@pytest.mark.parametrize("bf16,layout", [(True, 1), (False, 0)], ids=["bf16_rows", "f32"])
def test_gemm_many_rows_other_formats(hsd, bf16, layout):
    import torch
    m, n, k = 130, 600, 256
    rng = np.random.default_rng(77)
    x = rng.standard_normal((m, k)).astype(np.float32)
    w = (rng.standard_normal((n, k)) / np.sqrt(k)).astype(np.float32)
    if bf16:
        x, w = inputs.bf16_round(x), inputs.bf16_round(w)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    dt, td = (hsd.BF16, torch.bfloat16) if bf16 else (hsd.F32, torch.float32)
    got = hsd.gemm(_cuda(x, td), hsd.pack_weight(_cuda(w, td), dt, layout), n, dt, None, layout).cpu().numpy()
    assert np.abs(got - ref).max() < 4e-6 * np.sqrt(k) * np.abs(ref).max() + 1e-6


@pytest.mark.parametrize("group", [1, 2, 4, 8])
@pytest.mark.parametrize("m,n,k", [(1, 96, 32), (5, 200, 96), (3, 64, 7 * 32), (9, 130, 9 * 32), (16, 48, 130 * 32), (4, 2048, 4096),
                                   (33, 96, 11 * 32), (64, 160, 19 * 32)])
def test_gemm_wave_groups(hsd, m, n, k, group):
    """How the eight waves of a workgroup share its 32-wide k-steps (contiguous slices, or round-robin inside groups of
    2, 4 or 8 waves) must not change the product: k-step counts below, equal to and not divisible by the number of waves
    and groups, one to four row tiles, with and without a split of K over workgroups."""
    import torch
    rng = np.random.default_rng(m + n + k)
    x = inputs.bf16_round(rng.standard_normal((m, k)).astype(np.float32))
    w = inputs.bf16_round((rng.standard_normal((n, k)) / np.sqrt(k)).astype(np.float32))
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    packed = hsd.pack_weight(_cuda(w, torch.bfloat16), hsd.BF16)
    for ksplit in (0, 3):
        tn = hsd.kernel_tuning(gemm_interleave={0: group if group > 1 else -1}, gemm_ksplit={0: ksplit})
        got = hsd.gemm(_cuda(x, torch.bfloat16), packed, n, hsd.BF16, None, 0, tn).cpu().numpy()
        assert np.abs(got - ref).max() < 4e-6 * np.sqrt(k) * np.abs(ref).max() + 1e-6, (group, ksplit)


def test_gemm_split_k_exchange_repeated(hsd):
    """The split-K partial tiles travel through one reused workspace: 60 launches with fresh
    activations each must all match (a stale or early read of a partial would show up here)."""
    import torch
    m, n, k = 6, 2048, 2048                     # 128 column groups x 8 K slices
    rng = np.random.default_rng(5)
    w = inputs.bf16_round((rng.standard_normal((n, k)) / np.sqrt(k)).astype(np.float32))
    packed = hsd.pack_weight(_cuda(w, torch.bfloat16), hsd.BF16)
    ws = torch.zeros(hsd.lib.hsd_gemm_workspace_bytes(m, n, k), dtype=torch.uint8, device="cuda")
    w64 = w.astype(np.float64).T
    xs = [inputs.bf16_round(rng.standard_normal((m, k)).astype(np.float32) * (1 + i % 5)) for i in range(60)]
    outs = [hsd.gemm(_cuda(x, torch.bfloat16), packed, n, hsd.BF16, ws) for x in xs]      # queued back to back
    for i, (x, y) in enumerate(zip(xs, outs)):
        ref = x.astype(np.float64) @ w64
        assert np.abs(y.cpu().numpy() - ref).max() < 4e-6 * np.sqrt(k) * np.abs(ref).max() + 1e-6, i


# ---- k-query attention over the paged cache ------------------------------------------------------
def _attention_ref(q, k, v, pos0):
    """Textbook attention in fp64: q [B, m, n_q, hd], k / v [B, S, n_kv, hd] (S >= pos0 + m), causal among the
    m new tokens at positions pos0[b] + i.  One (sequence, KV head) at a time: scores of all its query rows as one
    matrix product, masked, row-wise softmax, times V."""
    B, m, n_q, hd = q.shape
    n_kv = k.shape[2]
    group = n_q // n_kv
    out = np.zeros(q.shape)
    for b in range(B):
        L = int(pos0[b]) + m
        for g in range(n_kv):
            kk = k[b, :L, g].astype(np.float64)
            vv = v[b, :L, g].astype(np.float64)
            qq = q[b, :, g * group:(g + 1) * group].astype(np.float64).reshape(m * group, hd)     # row = i * group + h
            sc = qq @ kk.T / np.sqrt(hd)
            limit = int(pos0[b]) + 1 + np.repeat(np.arange(m), group)                               # positions < limit visible
            sc[np.arange(L)[None, :] >= limit[:, None]] = -np.inf
            w = np.exp(sc - sc.max(axis=1, keepdims=True))
            out[b, :, g * group:(g + 1) * group] = ((w / w.sum(axis=1, keepdims=True)) @ vv).reshape(m, group, hd)
    return out


def _attention_ref_loops(q, k, v, pos0):
    """The same definition written as plain loops over (sequence, token, head); pins the vectorised form above."""
    B, m, n_q, hd = q.shape
    n_kv = k.shape[2]
    out = np.zeros(q.shape)
    for b in range(B):
        for i in range(m):
            L = int(pos0[b]) + i + 1
            for h in range(n_q):
                g = h // (n_q // n_kv)
                sc = k[b, :L, g].astype(np.float64) @ q[b, i, h].astype(np.float64) / np.sqrt(hd)
                w = np.exp(sc - sc.max())
                out[b, i, h] = (w / w.sum()) @ v[b, :L, g].astype(np.float64)
    return out


# Bound on max|got - ref| relative to max|ref| of the cell.  bf16: the stored output is rounded to bf16 (2^-9 of
# each value) and the probabilities enter the P V product rounded to bf16 (2^-9 each, averaging down over the
# positions); 1e-2 leaves a factor of about three.  fp32: a few ulps of the sums.
ATT_REL_TOL = {True: 1e-2, False: 2e-5}


def _attention_cell(hsd, B, S, ms, n_q, n_kv, hd, bf16, check_alt=True):
    """One cache of B ragged sequences of up to S positions behind a permuted page table; for each m in ms the last m
    positions of every sequence are the new tokens.  Returns nothing; asserts the relative bound per m."""
    import torch
    rng = np.random.default_rng(S + ms[0])
    rnd = (lambda sh: inputs.bf16_round(rng.standard_normal(sh, dtype=np.float32))) if bf16 else (lambda sh: rng.standard_normal(sh, dtype=np.float32))
    lens = [S - (b * 37) % max(1, S // 3) for b in range(B)]           # total positions per sequence, new tokens included
    k, v = rnd((B, S, n_kv, hd)), rnd((B, S, n_kv, hd))
    dt, td = (hsd.BF16, torch.bfloat16) if bf16 else (hsd.F32, torch.float32)
    max_pages = (S + 63) // 64
    perm = np.random.default_rng(1).permutation(B * max_pages)
    cache = hsd.KvLayer(B, S, n_kv, hd, dt, perm)
    zero = torch.zeros(B, dtype=torch.int32, device="cuda")
    # fill every sequence up to its own length (rows beyond stay zero), in two writes to exercise offsets
    n1 = min(lens) // 2
    cache.write(zero, _cuda(k[:, :n1], td), _cuda(v[:, :n1], td))
    for b in range(B):
        one = hsd.KvLayer.__new__(hsd.KvLayer)
        one.__dict__.update(cache.__dict__)
        one.batch = 1
        one.pages = cache.pages[b:b + 1].contiguous()
        one.write(torch.tensor([n1], dtype=torch.int32, device="cuda"), _cuda(k[b:b + 1, n1:lens[b]], td), _cuda(v[b:b + 1, n1:lens[b]], td))
    for m in ms:
        q = rnd((B, m, n_q, hd))
        pos0 = np.array([l - m for l in lens], dtype=np.int32)
        got = cache.attention(_cuda(q, td), _cuda(pos0), max(lens)).float().cpu().numpy()
        ref = _attention_ref(q, k, v, pos0)
        err, scale = np.abs(got - ref).max(), np.abs(ref).max()
        say("  B %d S %d m %d: max abs err %.2e, max |ref| %.3f, ratio %.2e" % (B, S, m, err, scale, err / scale))
        assert err <= ATT_REL_TOL[bf16] * scale, (B, S, m, err, scale)
        if check_alt and bf16 and m * (n_q // n_kv) > 16:
            # the two-tiles-per-workgroup variant (a tuning alternative) on the same inputs
            got2 = cache.attention(_cuda(q, td), _cuda(pos0), max(lens), tuning=hsd.kernel_tuning(attn_qt1_rows=16)).float().cpu().numpy()
            assert np.abs(got2 - ref).max() <= ATT_REL_TOL[bf16] * scale


def test_attention_reference_forms_agree():
    """CPU only in effect (no kernel runs): the vectorised reference equals the loop form on a ragged GQA case."""
    rng = np.random.default_rng(3)
    q, k, v = rng.standard_normal((2, 5, 6, 32)), rng.standard_normal((2, 90, 2, 32)), rng.standard_normal((2, 90, 2, 32))
    pos0 = np.array([85, 40], dtype=np.int32)
    assert np.abs(_attention_ref(q, k, v, pos0) - _attention_ref_loops(q, k, v, pos0)).max() < 1e-13


@pytest.mark.parametrize("B,S,m,n_q,n_kv,hd,bf16", [
    (1, 100, 1, 4, 4, 64, False), (2, 333, 5, 6, 2, 32, False),
    (1, 70, 1, 8, 8, 64, True), (1, 777, 6, 32, 8, 64, True), (3, 1500, 4, 8, 8, 128, True), (2, 4200, 16, 16, 2, 128, True),
    (1, 9000, 8, 8, 1, 64, True), (8, 300, 2, 4, 4, 128, True), (1, 640, 16, 32, 8, 64, True),
    (1, 32768, 4, 16, 4, 128, True),                       # the longest context of the microbenchmark configuration
])
def test_attention(hsd, B, S, m, n_q, n_kv, hd, bf16):
    """Per-sequence lengths differ (ragged batch), pages are permuted; error bounded relative to the largest output
    of the cell (outputs shrink like 1 / sqrt(positions) on random K/V, so an absolute bound would not bind)."""
    say("attention", B, S, m, n_q, n_kv, hd, "bf16" if bf16 else "f32")
    _attention_cell(hsd, B, S, [m], n_q, n_kv, hd, bf16)


@pytest.mark.parametrize("B,S,ms,n_q,n_kv,hd", [
    # the layer microbenchmark's shape (32 x 128 heads, no grouping): the sequence is split over workgroups and merged
    (1, 4096, (1, 4, 16), 32, 32, 128),
    (1, 16384, (1, 4, 16), 32, 32, 128),
    (8, 4096, (1, 4, 16), 32, 32, 128),
    (8, 16384, (4,), 32, 32, 128),
    # grouped heads of 64 dims at 8192 positions, and the widest target's head layout (64 query / 8 KV x 128) at its prompt length
    (1, 8192, (1, 6), 32, 8, 64),
    (1, 8448, (1, 4, 8), 64, 8, 128),
])
def test_attention_split_sequence_cells(hsd, B, S, ms, n_q, n_kv, hd):
    """Long contexts at the real head counts, where every launch splits the sequence over workgroups and merges the
    partial softmax states: bf16, ragged lengths, permuted pages, relative bound per cell."""
    say("attention (split sequence)", B, S, ms, n_q, n_kv, hd)
    _attention_cell(hsd, B, S, list(ms), n_q, n_kv, hd, True, check_alt=False)


def test_attention_random_cells(hsd):
    """Fourteen cells drawn at random: batch 1-5, 20-3000 cached positions, 1-24 new tokens, one to eight KV heads
    with one to eight query heads each, both head sizes, both storage types."""
    rng = np.random.default_rng(99)
    for _ in range(14):
        n_kv = int(rng.choice([1, 2, 4, 8]))
        group = int(rng.choice([1, 2, 4, 8]))
        m = int(rng.integers(1, 25))
        S = int(rng.integers(max(20, m + 3), 3000))
        bf16 = bool(rng.integers(0, 4))                       # mostly the MFMA path
        hd = int(rng.choice([64, 128])) if bf16 else int(rng.choice([32, 64, 96]))
        test_attention(hsd, int(rng.integers(1, 6)), S, m, n_kv * group, n_kv, hd, bf16)
