"""Pins for the oracle's uncertainty-driven measurement budget (Sec. 8.1), CPU only."""
import math
import numpy as np
import pytest
import scipy.stats
import oracle


def test_entropy_closed_forms():
    V = 1000
    assert oracle.softmax_entropy(np.zeros(V)) == pytest.approx(math.log(V), abs=1e-12)          # uniform
    assert oracle.softmax_entropy(np.full(V, 37.5)) == pytest.approx(math.log(V), abs=1e-12)     # shift invariance
    x = np.full(V, -1e9)
    x[7] = 0.0
    assert oracle.softmax_entropy(x) == pytest.approx(0.0, abs=1e-12)                            # one certain token
    a = 0.3
    two = np.full(V, -1e9)
    two[0], two[1] = math.log(a), math.log(1 - a)
    assert oracle.softmax_entropy(two) == pytest.approx(-(a * math.log(a) + (1 - a) * math.log(1 - a)), abs=1e-12)
    rng = np.random.default_rng(0)
    L = rng.standard_normal((5, 300)) * 3
    p = np.exp(L - L.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    assert np.allclose(oracle.softmax_entropy(L), scipy.stats.entropy(p, axis=1), atol=1e-12)    # library routine
    assert oracle.softmax_entropy(L + 100.0)[2] == pytest.approx(oracle.softmax_entropy(L)[2], abs=1e-10)


def test_budget_hand_examples_and_clipping():
    # m_base (1 + gamma H): 128 * (1 + 0.25 * 2.0) = 192
    assert oracle.uds_budget(128, 0.25, 2.0, 64, 512) == 192
    assert oracle.uds_budget(128, 0.25, 0.0, 64, 512) == 128                # confident step: the base budget
    assert oracle.uds_budget(128, 0.25, 2.03, 64, 512) == 192               # floor(192.96)
    assert oracle.uds_budget(128, 0.25, 20.0, 64, 512) == 512               # clipped above
    assert oracle.uds_budget(32, 0.25, 0.0, 64, 512) == 64                  # clipped below
    assert oracle.uds_budget(100, 0.1, math.log(32000), 64, 512) == math.floor(100 * (1 + 0.1 * math.log(32000)))
    m = [oracle.uds_budget(128, 0.25, h, 64, 512) for h in np.linspace(0, 12, 50)]
    assert all(b >= a for a, b in zip(m, m[1:]))                            # monotone in the entropy
    with pytest.raises(ValueError):
        oracle.uds_budget(128, 0.25, 1.0, 600, 512)


def test_library_budget_function_matches_the_oracle():
    """cs_uds_budget is host arithmetic: it can be checked without a GPU."""
    from paper_2604_14156_amd import binding
    lib = binding.load_library()
    rng = np.random.default_rng(1)
    for _ in range(200):
        m_base = int(rng.integers(1, 600))
        gamma = float(np.float32(rng.uniform(0, 1)))
        H = float(np.float32(rng.uniform(0, 12)))
        lo = int(rng.integers(1, 300))
        hi = lo + int(rng.integers(0, 600))
        assert lib.cs_uds_budget(m_base, gamma, H, lo, hi) == oracle.uds_budget(m_base, gamma, H, lo, hi)
    assert lib.cs_uds_budget(128, 0.25, 1.0, 600, 512) == -1
    assert lib.cs_uds_budget(128, 0.25, float("nan"), 64, 512) == -1
    assert lib.cs_uds_budget(128, 0.25, 1.0, 0, 512) == -1
