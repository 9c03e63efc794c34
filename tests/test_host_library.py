"""CPU-only checks of libhsd.so: it loads, exports every entry point the header declares, and its
host-side latency model / hierarchy selection agree with the oracle (no GPU work is issued)."""
import os
import re

import numpy as np
import pytest

from oracle import latency
from paper_2510_19705_amd import hsd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "hsd.h")).read() + open(os.path.join(ROOT, "include", "hsd_dev.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(hsd_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 30
    for name in sorted(declared):
        assert hasattr(hsd.lib, name), name
    assert declared == set(hsd.EXPORTS), declared ^ set(hsd.EXPORTS)


def test_gamma_matches_oracle():
    rng = np.random.default_rng(0)
    for _ in range(200):
        a, ti, tj = float(rng.uniform(0, 1)), int(rng.integers(1, 16)), int(rng.integers(1, 16))
        assert abs(hsd.gamma(a, ti, tj) - latency.gamma(a, ti, tj)) < 1e-12
    assert hsd.gamma(1.5, 1, 1) < 0 and hsd.gamma(0.5, 0, 1) < 0


def test_expected_latency_matches_oracle():
    rng = np.random.default_rng(1)
    for _ in range(100):
        K = int(rng.integers(0, 5))
        c = rng.uniform(0.1, 10, K + 1).tolist()
        a = rng.uniform(0, 1, K).tolist()
        T = [int(v) for v in rng.integers(1, 8, K)]
        assert abs(hsd.expected_latency(c, a, T) - latency.latency_literal(c, a, T)) < 1e-10
        assert abs(hsd.expected_latency(c, a, T, True) - latency.latency_exact(c, a, T)) < 1e-10
    assert hsd.expected_latency([1.0, -2.0], [0.5], [1]) < 0


@pytest.mark.parametrize("monotone", [True, False])
def test_select_hierarchy_matches_oracle(monotone):
    rng = np.random.default_rng(2)
    for _ in range(25):
        n = int(rng.integers(1, 7))
        cost = sorted(rng.uniform(0.01, 2.0, n - 1).tolist()) + [float(rng.uniform(5, 40))]
        alpha = np.triu(rng.uniform(0.05, 0.95, (n, n)), 1)
        lat, sig, T = hsd.select_hierarchy(cost, alpha, 8, monotone)
        ref = latency.select_hierarchy(cost, alpha.tolist(), 8, monotone)
        assert abs(lat - ref[0]) < 1e-10 and sig == ref[1] and T == ref[2]
        b = hsd.best_single_draft(cost, alpha, 8)
        rb = latency.best_single_draft(cost, alpha.tolist(), 8)
        assert abs(b[0] - rb[0]) < 1e-10 and (b[1], b[2]) == ((-1, 0) if rb[1] is None else (rb[1], rb[2]))


def test_select_hierarchy_printed_example():
    """Sec. 3.4 table, two models: c = (4, 33), alpha = 0.8 -> T = 5, latency 14.37 (2.2971x)."""
    lat, sig, T = hsd.select_hierarchy([4.0, 33.0], [[0, 0.8], [0, 0]], 15)
    assert sig == [0, 1] and T == [5] and abs(lat - 14.37) < 0.005 and abs(33.0 / lat - 2.2971) < 1e-4


def test_select_hierarchy_rejects_bad_input():
    with pytest.raises(hsd.HsdError):
        hsd.select_hierarchy([1.0, 0.0], [[0, 0.5], [0, 0]], 4)
    with pytest.raises(hsd.HsdError):
        hsd.select_hierarchy([1.0, 2.0], [[0, 1.5], [0, 0]], 4)
    with pytest.raises(hsd.HsdError):
        hsd.select_hierarchy([1.0, 2.0], [[0, 0.5], [0, 0]], 0)


def test_size_helpers_and_descriptor_validation():
    """Pure host arithmetic: no device is touched."""
    import ctypes as C
    d = hsd.ModelDesc(2, 64, 4, 2, 32, 128, 100, hsd.BF16, 10000.0, 1e-5, 128, 16)
    assert hsd.lib.hsd_model_weight_bytes(C.byref(d)) % 256 == 0 and hsd.lib.hsd_model_weight_bytes(C.byref(d)) > 0
    assert hsd.lib.hsd_model_kv_bytes(C.byref(d)) == 2 * (128 // 64) * 2 * 2 * 64 * 32 * 2
    bad = hsd.ModelDesc(2, 64, 4, 3, 32, 128, 100, hsd.BF16, 10000.0, 1e-5, 128, 16)      # n_q % n_kv != 0
    assert hsd.lib.hsd_model_weight_bytes(C.byref(bad)) == 0 and b"n_q" in hsd.lib.hsd_last_error()
    bad = hsd.ModelDesc(2, 64, 4, 2, 32, 128, 100, hsd.BF16, 10000.0, 1e-5, 100, 16)      # max_seq not a page multiple
    assert hsd.lib.hsd_model_kv_bytes(C.byref(bad)) == 0
    assert hsd.lib.hsd_packed_bytes(100, 64, hsd.BF16) == 112 * 64 * 2
    assert hsd.lib.hsd_sampler_scratch_bytes(128256) >= 16 + 2 * 63 * 8
