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


@pytest.mark.parametrize("chain", [False, True], ids=["noise_from_target", "noise_chain"])
def test_distilled_study_runs_on_the_small_configuration(chain):
    """Synthetic closeness on the stand-in configuration: every run generates the tokens asked for, fixed-cost prices
    are positive, acceptance rates are frequencies, and with a chain of noise steps neighbouring candidates accept
    more than the two ends of the chain."""
    from paper_2510_19705_amd import workloads
    out = workloads.run_distilled("smoke", [0.8, 0.3], gen=48, chain=chain)
    runs = out["runs"]
    assert {"autoregressive", "selected"} <= set(runs)
    for key, r in runs.items():
        assert r["tokens"] >= 48 and r["artificial_ms_per_token"] > 0, key
        assert all(0 <= a <= 1 for a in r["per_test_acceptance"]), key
    alpha = np.array(out["alpha"])
    assert np.allclose(alpha, alpha.T) and np.allclose(np.diag(alpha), 1)
    if chain:
        assert alpha[1, 2] > alpha[0, 2]                    # one noise step against two
    assert out["selected_vs_best_single_draft"] > 0
