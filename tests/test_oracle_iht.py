"""Pins for the oracle's block iterative hard thresholding (CPU only)."""
import itertools
import numpy as np
import pytest
import oracle
from paper_2604_14156_amd import workloads as wl


def test_orthonormal_dictionary_one_step_is_exact():
    rng = np.random.default_rng(1)
    G = m = 20
    Q, _ = np.linalg.qr(rng.standard_normal((m, G)))
    Q = Q[:, :G]
    y = rng.standard_normal(m)
    c = Q.T @ y
    k = 6
    top = np.sort(np.argsort(-np.abs(c), kind="stable")[:k])
    # k*rb < m is required, so use 19 columns
    Q19 = Q[:, :19]
    c19 = Q19.T @ y
    top19 = np.sort(np.argsort(-np.abs(c19), kind="stable")[:k])
    for iters in (1, 3):
        rec = oracle.block_iht(Q19, y, 19, 1, k, iters, True)
        assert list(rec["support"]) == list(top19)
        assert np.allclose(rec["coef"], c19[top19], atol=1e-12)
    srt = np.sort(c19 ** 2)[::-1]
    assert abs(rec["margin"] - (srt[k - 1] - srt[k]) / srt[k - 1]) < 1e-10
    assert len(top) == k


def test_planted_solution_is_a_fixed_point_and_is_reached():
    rng = np.random.default_rng(2)
    G, m, k = 64, 48, 6
    M = rng.standard_normal((m, G)) / np.sqrt(m)
    for trial in range(5):
        S = np.sort(rng.choice(G, size=k, replace=False))
        alpha = np.zeros(G)
        alpha[S] = rng.choice([-1.0, 1.0], size=k) * rng.uniform(1.0, 2.0, size=k)
        y = M @ alpha
        rec = oracle.block_iht(M, y, G, 1, k, 30, True)
        assert list(rec["support"]) == list(S)
        assert np.allclose(rec["coef"], alpha[S], atol=1e-9)
        assert rec["resid_norm"] < 1e-10


def test_tiny_instances_against_brute_force():
    rng = np.random.default_rng(3)
    G, m, k = 10, 24, 3
    hits = 0
    for trial in range(10):
        M = rng.standard_normal((m, G)) / np.sqrt(m)
        S = np.sort(rng.choice(G, size=k, replace=False))
        alpha = np.zeros(G)
        alpha[S] = rng.choice([-1.0, 1.0], size=k) * rng.uniform(2.0, 3.0, size=k)
        y = M @ alpha + 1e-3 * rng.standard_normal(m)
        best, best_set = np.inf, None
        for T in itertools.combinations(range(G), k):
            co, *_ = np.linalg.lstsq(M[:, T], y, rcond=None)
            res = np.linalg.norm(y - M[:, T] @ co)
            if res < best:
                best, best_set = res, T
        rec = oracle.block_iht(M, y, G, 1, k, 20, True)
        assert rec["resid_norm"] >= best - 1e-12            # never better than the optimum
        hits += tuple(rec["support"]) == best_set == tuple(S)
    assert hits >= 9


def test_first_step_matches_an_explicit_line_search():
    rng = np.random.default_rng(4)
    G, m, k = 30, 40, 5
    M = rng.standard_normal((m, G))
    y = rng.standard_normal(m)
    w = np.linalg.norm(M, axis=0)
    g = M.T @ y
    S0 = np.sort(np.argsort(-(w * g) ** 2, kind="stable")[:k])
    gs = np.zeros(G); gs[S0] = g[S0]
    # mu minimises ||y - mu M g_S||: scan a fine grid around the closed form
    mu_closed = (gs @ gs) / np.sum((M @ gs) ** 2)
    grid = mu_closed * np.linspace(0.5, 1.5, 2001)
    mu_best = grid[np.argmin([np.linalg.norm(y - mu * (M @ gs)) for mu in grid])]
    assert abs(mu_best - mu_closed) <= 1e-3 * mu_closed
    p = mu_closed * g
    S1 = np.sort(np.argsort(-(w * p) ** 2, kind="stable")[:k])
    rec = oracle.block_iht(M, y, G, 1, k, 1, True)
    assert list(rec["support"]) == list(S1)
    ref, *_ = np.linalg.lstsq(M[:, S1], y, rcond=None)
    assert np.allclose(rec["coef"], ref, atol=1e-10)
    assert np.abs(M[:, S1].T @ rec["residual"]).max() < 1e-10


def test_block_units_and_weighting():
    rng = np.random.default_rng(5)
    G, rb, m, k = 12, 2, 40, 3
    M = rng.standard_normal((m, G * rb)) * rng.uniform(0.2, 5.0, size=G * rb)
    S = np.sort(rng.choice(G, size=k, replace=False))
    alpha = np.zeros(G * rb)
    for g in S:
        alpha[g * rb:(g + 1) * rb] = rng.standard_normal(rb) * 3.0 / np.linalg.norm(M[:, g * rb:(g + 1) * rb], axis=0)
    y = M @ alpha
    rec = oracle.block_iht(M, y, G, rb, k, 40, True)
    assert list(rec["support"]) == list(S)
    assert rec["resid_norm"] < 1e-8 * np.linalg.norm(y)
    with pytest.raises(ValueError):
        oracle.block_iht(M, y, G, rb, 20, 3, True)          # k*rb >= m
    with pytest.raises(ValueError):
        oracle.block_iht(M, y, G, rb, k, 0, True)


def test_decode_shape_quality_is_close_to_greedy_pursuit():
    c = wl.CFG2
    seed = 2000
    rng = wl.rng_for(seed)
    pi, psi = wl.make_profiles(rng, c.G, c.b)
    z, S = wl.plant_usage(rng, pi, c.k, 4, c.amp, c.bg)
    M = oracle.effective_matrix(c.ens, seed, 4, c.m, c.n, c.G, c.b, 1, psi)
    Y = oracle.sketch(c.ens, seed, 4, c.m, z)
    ov_iht = ov_omp = 0
    for t in range(4):
        a = oracle.block_iht(M, Y[t], c.G, 1, c.k, 12, True)
        b = oracle.block_omp(M, Y[t], c.G, 1, c.k, True)
        ov_iht += len(set(a["support"]) & set(S[t]))
        ov_omp += len(set(b["support"]) & set(S[t]))
    assert ov_iht >= 0.9 * ov_omp


def test_the_iteration_stops_once_the_fit_on_the_support_is_reached():
    """Past convergence the line search is a quotient of two rounding errors; the iteration ends when the
    gradient on the support has dropped to 1e-3 of its first value, so more iterations change nothing: same
    support, and the margin is that of the last projection that was made (a well-defined number, the same
    for every iteration count past convergence)."""
    rng = np.random.default_rng(12)
    G, m, k = 12, 72, 2
    M = rng.standard_normal((m, G)) / np.sqrt(m)
    S = np.array([3, 8])
    y = M[:, S] @ np.array([1.5, -1.0]) + 0.05 * rng.standard_normal(m)
    recs = [oracle.block_iht(M, y, G, 1, k, iters, True) for iters in (20, 21, 50, 400)]
    for r in recs[1:]:
        assert list(r["support"]) == list(recs[0]["support"]) == list(S)
        assert r["margin"] == recs[0]["margin"]
    # the margin that stands is a projection's gap, strictly inside (0, 1): off-support units have energy there
    assert 0.0 < recs[0]["margin"] < 1.0
    # an orthonormal dictionary converges in one step: the second iteration already stops
    Q, _ = np.linalg.qr(rng.standard_normal((m, G)))
    one, many = oracle.block_iht(Q, y, G, 1, k, 1, True), oracle.block_iht(Q, y, G, 1, k, 9, True)
    assert list(one["support"]) == list(many["support"]) and one["margin"] == many["margin"]
