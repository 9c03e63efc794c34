"""The large-shape workload script on its small stand-in configuration: runs end to end on the GPU and its numbers
are self-consistent (the real configurations differ only in shapes)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_smoke_configuration_runs():
    from paper_2510_19705_amd import workloads
    out = workloads.run("smoke")
    n = len(out["candidates"])
    alpha = np.array(out["alpha"])
    assert alpha.shape == (n, n) and np.allclose(alpha, alpha.T) and np.allclose(np.diag(alpha), 1)
    assert ((alpha > 0) & (alpha <= 1 + 1e-9)).all()
    assert alpha[1, 2] > alpha[0, 2]                        # an early exit of the target agrees more than a foreign network
    assert len(out["cost_ms"]) == n and all(c > 0 for c in out["cost_ms"])
    sel = out["selected"]
    assert sel["levels"][-1] == out["candidates"][-1]       # the target is always the last level
    m = out["measured"]
    assert m["autoregressive"]["tokens_per_s"] > 0
    for key, r in m.items():
        if "error" not in r:
            assert r["tokens_per_s"] > 0 and r["passes"][-1] > 0, key
    for p in out["verify_pass"].values():
        assert 0 < p["hbm_frac"] < 1
