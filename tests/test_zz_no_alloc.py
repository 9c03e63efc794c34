"""hsd_accept_resample_static (the sampler entry point that allocates nothing: its ticket and slice totals live in an
array built into the library) against hsd_accept_resample with a caller's scratch buffer, bit for bit, and against
the oracle's Verify; two calls in a row on the shared array, the second on a smaller vocabulary."""
import numpy as np
import pytest

from oracle import specsample
from paper_2510_19705_amd import inputs
from helpers import say

pytestmark = pytest.mark.gpu


def _cuda(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_static_scratch_sampler_matches_workspace_sampler():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2510_19705_amd import hsd
    seed = 0x5EED0001
    # both vocabularies above 32768, so that the multi-workgroup kernel (the one with a scratch buffer) runs; the
    # second call is smaller than the first and finds the first call's totals still in the array
    cases = [(128256, 6, 0), (40961, 3, 1), (128256, 0, 2), (50000, 16, 3), (2048, 4, 4)]
    for V, t, call in cases:
        say("accept_resample_static", V, t, call)
        p, q, x = inputs.make_prob_rows(V, t, seed=31 * V + t, sigma=3.0, noise=0.7)
        ref = specsample.verify(list(p), list(q), list(x), specsample.PhiloxChooser(seed), level=1, call=call)
        pd, qd = _cuda(p), (_cuda(q) if t else _cuda(p[:0]))
        x1 = _cuda(np.concatenate([x, [0]]).astype(np.int32))
        x2 = x1.clone()
        res = hsd.accept_resample_static(pd, qd, x1, seed, 1, call)
        torch.cuda.synchronize()
        n, m = res.cpu().tolist()
        got2 = hsd.accept_resample(pd, qd, x2, seed, 1, call)
        assert (n, m) == got2, (V, t, (n, m), got2)
        assert (n, m) == ref, (V, t, (n, m), ref)
        assert torch.equal(x1, x2) and int(x1[n].item()) == m


def test_static_scratch_sampler_back_to_back_on_one_stream():
    """Several calls queued without a synchronisation between them share the array in stream order."""
    import torch
    from paper_2510_19705_amd import hsd
    seed = 0x5EED0002
    sizes = [(70000, 5), (33000, 2), (128256, 9), (36000, 1)]
    held = []
    for call, (V, t) in enumerate(sizes):
        p, q, x = inputs.make_prob_rows(V, t, seed=7 * V + t, sigma=2.0, noise=0.5)
        pd, qd = _cuda(p), _cuda(q)
        xd = _cuda(np.concatenate([x, [0]]).astype(np.int32))
        held.append((p, q, x, pd, qd, xd, None))
    torch.cuda.synchronize()
    out = []
    for call, (p, q, x, pd, qd, xd, _) in enumerate(held):
        out.append(hsd.accept_resample_static(pd, qd, xd, seed, 2, call))
    torch.cuda.synchronize()
    for call, ((p, q, x, pd, qd, xd, _), res) in enumerate(zip(held, out)):
        ref = specsample.verify(list(p), list(q), list(x), specsample.PhiloxChooser(seed), level=2, call=call)
        assert tuple(res.cpu().tolist()) == ref, (call, res.cpu().tolist(), ref)


def test_static_scratch_sampler_rejects_what_it_cannot_hold():
    import torch
    from paper_2510_19705_amd import hsd
    V = 262144 + 1
    p = torch.zeros((1, 8), dtype=torch.float32, device="cuda")         # never read: the size check comes first
    x = torch.zeros(1, dtype=torch.int32, device="cuda")
    res = torch.zeros(2, dtype=torch.int32, device="cuda")
    rc = hsd.lib.hsd_accept_resample_static(p.data_ptr(), None, x.data_ptr(), 0, V, 1, 0, 0, res.data_ptr(), hsd._stream())
    assert rc == -2 and b"vocabulary" in hsd.lib.hsd_last_error()
