"""Pins for the oracle's block-OMP (CPU only): brute force, closed forms, the
incoherence guarantee (Prop. 1), noiseless exactness (Thm. 1), the measurement
scaling of Thm. 2 and a library least-squares routine."""
import itertools
import math
import numpy as np
import pytest
import oracle
from oracle import GAUSS
from paper_2604_14156_amd import workloads as wl


def _brute_force(M, y, G, rb, k):
    best, best_set = np.inf, None
    for S in itertools.combinations(range(G), k):
        cols = np.concatenate([np.arange(g * rb, (g + 1) * rb) for g in S])
        coef, *_ = np.linalg.lstsq(M[:, cols], y, rcond=None)
        res = np.linalg.norm(y - M[:, cols] @ coef)
        if res < best:
            best, best_set = res, S
    return best, best_set


def _cfg1_instance(seed):
    c = wl.CFG1
    rng = wl.rng_for(seed)
    pi, psi = wl.make_profiles(rng, c.G, c.b)
    z, S = wl.plant_usage(rng, pi, c.k, 1, c.amp, c.bg)
    noise = c.noise * rng.standard_normal(c.m)
    M = oracle.effective_matrix(c.ens, seed, 0, c.m, c.n, c.G, c.b, 1, psi)
    y = oracle.sketch(c.ens, seed, 0, c.m, z[0]) + noise
    return M, y, S[0]


def test_omp_equals_brute_force_on_tiny_planted_instances():
    c = wl.CFG1
    assert math.comb(c.G, c.k) == 1820
    for seed in (1000, 1001, 1002):
        M, y, S_true = _cfg1_instance(seed)
        rec = oracle.block_omp(M, y, c.G, 1, c.k, True)
        best, best_set = _brute_force(M, y, c.G, 1, c.k)
        assert tuple(rec["support"]) == best_set == tuple(S_true)
        assert abs(rec["resid_norm"] - best) < 1e-10


def test_omp_residual_never_beats_brute_force():
    rng = np.random.default_rng(7)
    for _ in range(10):
        G, k, m = 10, 3, 12
        M = rng.standard_normal((m, G))
        y = rng.standard_normal(m)                     # nothing planted
        rec = oracle.block_omp(M, y, G, 1, k, True)
        best, _ = _brute_force(M, y, G, 1, k)
        assert rec["resid_norm"] >= best - 1e-12


def test_orthonormal_dictionary_closed_form():
    rng = np.random.default_rng(8)
    G = m = 24
    Q, _ = np.linalg.qr(rng.standard_normal((m, G)))
    y = rng.standard_normal(m)
    c = Q.T @ y
    k = 5
    rec = oracle.block_omp(Q, y, G, 1, k, True)
    top = np.sort(np.argsort(-np.abs(c), kind="stable")[:k])
    assert list(rec["support"]) == list(top)
    assert np.allclose(rec["coef"], c[top], atol=1e-12)
    rest = np.setdiff1d(np.arange(G), top)
    assert abs(rec["resid_norm"] - np.linalg.norm(c[rest])) < 1e-12
    # selection order follows |c| descending, and the margin is the smallest relative gap
    order = np.argsort(-np.abs(c), kind="stable")[:k + 1]
    assert list(rec["order"]) == list(order[:k])
    e = c[order] ** 2
    assert abs(rec["margin"] - min((e[i] - e[i + 1]) / e[i] for i in range(k))) < 1e-10


def test_single_unit_is_argmax_of_normalised_correlation():
    rng = np.random.default_rng(9)
    M = rng.standard_normal((20, 30)) * rng.uniform(0.1, 10.0, size=30)   # wildly different norms
    y = rng.standard_normal(20)
    rec = oracle.block_omp(M, y, 30, 1, 1, True)
    corr = np.abs(M.T @ y) / np.linalg.norm(M, axis=0)
    assert rec["support"][0] == int(np.argmax(corr))
    raw = oracle.block_omp(M, y, 30, 1, 1, False)
    assert raw["support"][0] == int(np.argmax(np.abs(M.T @ y)))


def test_incoherence_guarantee():
    """Prop. 1: k < (1 + 1/mu)/2 implies exact support recovery, noiseless."""
    rng = np.random.default_rng(10)
    checked = 0
    for trial in range(6):
        G, m = 16, 1024
        M = oracle.phi_matrix(GAUSS, 500 + trial, 0, m, G)
        Mn = M / np.linalg.norm(M, axis=0)
        gram = np.abs(Mn.T @ Mn)
        np.fill_diagonal(gram, 0.0)
        mu = gram.max()
        kmax = math.ceil(0.5 * (1.0 + 1.0 / mu)) - 1          # largest k strictly below the bound
        assert kmax >= 3
        for k in range(1, kmax + 1):
            S = np.sort(rng.choice(G, size=k, replace=False))
            alpha = np.zeros(G)
            alpha[S] = rng.choice([-1.0, 1.0], size=k) * rng.uniform(0.01, 100.0, size=k)
            rec = oracle.block_omp(M, M @ alpha, G, 1, k, True)
            assert list(rec["support"]) == list(S)
            assert np.allclose(rec["coef"], alpha[S], rtol=1e-9)
            assert rec["resid_norm"] < 1e-10 * np.linalg.norm(alpha)
            checked += 1
    assert checked >= 18


def test_noiseless_exactness():
    """Thm. 1, last sentence: sigma = eta = 0 gives exact recovery."""
    c = wl.CFG1
    for seed in (2000, 2001):
        rng = wl.rng_for(seed)
        pi, psi = wl.make_profiles(rng, c.G, c.b)
        z, S = wl.plant_usage(rng, pi, c.k, 1, "unit", 0.0)
        # the stored inputs are fp32; rebuild the dictionary in fp64 from the planted
        # vector itself so that z lies exactly in its span
        psi64 = np.array(psi, dtype=np.float64)
        for g in S[0]:
            blk = z[0, g * c.b:(g + 1) * c.b].astype(np.float64)
            psi64[g, :, 0] = blk / np.linalg.norm(blk)
        M = oracle.effective_matrix(c.ens, seed, 0, c.m, c.n, c.G, c.b, 1, psi64)
        y = oracle.sketch(c.ens, seed, 0, c.m, z[0])
        rec = oracle.block_omp(M, y, c.G, 1, c.k, True)
        assert list(rec["support"]) == list(S[0])
        assert rec["resid_norm"] < 1e-12 * np.linalg.norm(y)
        want = [np.linalg.norm(z[0, g * c.b:(g + 1) * c.b].astype(np.float64)) for g in S[0]]
        assert np.allclose(rec["coef"], want, rtol=1e-10)


def test_refit_matches_library_lstsq_and_is_orthogonal():
    rng = np.random.default_rng(11)
    G, rb, m, k = 12, 3, 40, 4
    M = rng.standard_normal((m, G * rb))
    y = rng.standard_normal(m)
    for normalised in (True, False):
        rec = oracle.block_omp(M, y, G, rb, k, normalised)
        cols = np.concatenate([np.arange(g * rb, (g + 1) * rb) for g in rec["support"]])
        ref, *_ = np.linalg.lstsq(M[:, cols], y, rcond=None)
        assert np.allclose(rec["coef"], ref, atol=1e-10)
        assert np.abs(M[:, cols].T @ rec["residual"]).max() < 1e-10
        assert abs(rec["resid_norm"] - np.linalg.norm(y - M[:, cols] @ ref)) < 1e-12


def test_textbook_block_mode_against_brute_force():
    """Identity dictionary, rb = b, on a well-posed shape (k*b < m)."""
    G, b, k, m = 8, 4, 2, 24
    rng = np.random.default_rng(12)
    for seed in range(4):
        M = oracle.effective_matrix(GAUSS, 3000 + seed, 1, m, G * b, G, b, b, None)
        S = np.sort(rng.choice(G, size=k, replace=False))
        z = np.zeros(G * b)
        for g in S:
            z[g * b:(g + 1) * b] = rng.standard_normal(b) + 3.0
        y = M @ z + 1e-3 * rng.standard_normal(m)
        rec = oracle.block_omp(M, y, G, b, k, False)
        best, best_set = _brute_force(M, y, G, b, k)
        assert tuple(rec["support"]) == best_set == tuple(S)
        assert abs(rec["resid_norm"] - best) < 1e-10


def test_block_score_uses_the_subspace_projection_when_normalised():
    # one unit with two nearly parallel columns: raw energy double counts, the projection does not
    m = 30
    rng = np.random.default_rng(13)
    a = rng.standard_normal(m)
    a /= np.linalg.norm(a)
    other = np.linalg.qr(rng.standard_normal((m, 2)))[0]
    M = np.column_stack([a, a + 1e-3 * other[:, 0], other[:, 0], other[:, 1]])   # units {0,1},{2,3}
    y = 1.0 * a + 1.2 * other[:, 1]
    assert oracle.block_omp(M, y, 2, 2, 1, False)["support"][0] == 0     # raw: 2*1 > 1.44
    assert oracle.block_omp(M, y, 2, 2, 1, True)["support"][0] == 1      # projected: 1 < 1.44


def test_ill_posed_and_range_errors():
    M = np.zeros((8, 16))
    with pytest.raises(ValueError):
        oracle.block_omp(M, np.zeros(8), 16, 1, 8, True)        # k*rb >= m
    with pytest.raises(ValueError):
        oracle.block_omp(M, np.zeros(8), 16, 1, 0, True)
    with pytest.raises(ValueError):
        oracle.block_omp(M, np.zeros(8), 8, 1, 2, True)         # column count mismatch


def _m50(G, k, rng, trials=24):
    """Smallest m on a grid with >= 50% exact recovery (Gaussian M, flat +-1 alpha)."""
    unit = k * math.log(math.e * G / k)
    for ratio in np.arange(0.6, 4.01, 0.2):
        m = max(k + 1, int(round(ratio * unit)))
        ok = 0
        for _ in range(trials):
            M = rng.standard_normal((m, G)) / math.sqrt(m)
            S = np.sort(rng.choice(G, size=k, replace=False))
            alpha = np.zeros(G)
            alpha[S] = rng.choice([-1.0, 1.0], size=k)
            ok += list(oracle.block_omp(M, M @ alpha, G, 1, k, True)["support"]) == list(S)
        if ok >= trials / 2:
            return m, ratio
    return None, None


def test_measurement_scaling_follows_k_log_G_over_k():
    """Thm. 2: the number of measurements for reliable recovery grows like
    k log(eG/k); the empirical 50% point divided by that unit stays within a
    narrow band over a range of G and k, and far below it recovery fails."""
    rng = np.random.default_rng(14)
    ratios = []
    for G, k in ((64, 4), (128, 4), (256, 4), (64, 8), (128, 8)):
        m50, ratio = _m50(G, k, rng)
        assert m50 is not None
        ratios.append(ratio)
    assert max(ratios) / min(ratios) <= 1.8
    # well below the transition nothing is recovered; well above, everything is
    G, k = 128, 8
    unit = k * math.log(math.e * G / k)
    for ratio, want in ((0.35, 0.0), (4.0, 1.0)):
        m = max(k + 1, int(ratio * unit))
        ok = 0
        for _ in range(12):
            M = rng.standard_normal((m, G)) / math.sqrt(m)
            S = np.sort(rng.choice(G, size=k, replace=False))
            alpha = np.zeros(G)
            alpha[S] = rng.choice([-1.0, 1.0], size=k)
            ok += list(oracle.block_omp(M, M @ alpha, G, 1, k, True)["support"]) == list(S)
        assert abs(ok / 12 - want) <= 0.2
