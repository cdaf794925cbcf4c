"""Pins for the oracle's warm-started (incremental) recovery (CPU only).

The procedure is a reading of Sec. 5 (temporal regulariser) and of the incremental
proposition of Sec. 10; it is pinned by its two limits (swaps = k is the greedy
solver, swaps = 0 a library least-squares fit), by brute force over every support
the drift budget allows, by closed forms of the regularised refit, and by the
measurement saving the proposition predicts.
"""
import itertools
import numpy as np
import pytest
import oracle


def _planted(rng, G, m, k, lo=1.0, hi=2.0):
    M = rng.standard_normal((m, G)) / np.sqrt(m)
    S = np.sort(rng.choice(G, size=k, replace=False))
    alpha = np.zeros(G)
    alpha[S] = rng.choice([-1.0, 1.0], size=k) * rng.uniform(lo, hi, size=k)
    return M, S, alpha


def _drift(rng, S, G, swaps):
    """Replace `swaps` units of S by units outside S."""
    S = list(S)
    out = rng.choice(len(S), size=swaps, replace=False)
    pool = [g for g in range(G) if g not in S]
    new = rng.choice(pool, size=swaps, replace=False)
    T = [g for i, g in enumerate(S) if i not in set(out.tolist())] + [int(g) for g in new]
    return np.sort(np.array(T))


def test_support_drift_metric_hand_examples():
    assert oracle.support_drift([1, 2, 3], [1, 2, 3]) == 0.0
    assert oracle.support_drift([1, 2, 3], [4, 5, 6]) == 1.0
    assert oracle.support_drift([1, 2, 3, 4], [1, 2, 3, 9]) == pytest.approx(2 / 5)     # {4,9} over {1,2,3,4,9}
    assert oracle.support_drift([], []) == 0.0


def test_full_budget_is_the_greedy_solver():
    rng = np.random.default_rng(11)
    G, m, k = 40, 32, 6
    for trial in range(4):
        M, S, alpha = _planted(rng, G, m, k)
        y = M @ alpha + 0.05 * rng.standard_normal(m)
        prev = rng.choice(G, size=k, replace=False)
        for normalised in (True, False):
            ref = oracle.block_omp(M, y, G, 1, k, normalised)
            rec = oracle.incremental_block_omp(M, y, G, 1, k, prev, k, normalised)
            assert list(rec["support"]) == list(ref["support"])
            assert rec["added"] == list(ref["order"])
            assert np.allclose(rec["coef"], ref["coef"], atol=1e-12)
            assert rec["margin"] == pytest.approx(ref["margin"], abs=1e-12)


def test_zero_budget_is_a_library_least_squares_fit_on_the_previous_support():
    rng = np.random.default_rng(12)
    G, m, k = 30, 24, 5
    M, S, alpha = _planted(rng, G, m, k)
    y = M @ alpha + 0.1 * rng.standard_normal(m)
    prev = np.array([7, 3, 22, 15, 9])
    rec = oracle.incremental_block_omp(M, y, G, 1, k, prev, 0, True)
    srt = np.sort(prev)
    co, *_ = np.linalg.lstsq(M[:, srt], y, rcond=None)
    assert list(rec["support"]) == list(srt)
    assert np.allclose(rec["coef"], co, atol=1e-12)
    assert rec["resid_norm"] == pytest.approx(np.linalg.norm(y - M[:, srt] @ co), abs=1e-12)
    assert rec["margin"] == 1.0 and rec["dropped"] == [] and rec["added"] == []


def test_blocks_of_two_atoms_reduce_to_the_same_limits():
    rng = np.random.default_rng(13)
    G, rb, m, k = 12, 2, 30, 3
    M = rng.standard_normal((m, G * rb)) / np.sqrt(m)
    y = rng.standard_normal(m)
    prev = [1, 5, 9]
    ref = oracle.block_omp(M, y, G, rb, k, True)
    rec = oracle.incremental_block_omp(M, y, G, rb, k, prev, k, True)
    assert list(rec["support"]) == list(ref["support"]) and np.allclose(rec["coef"], ref["coef"], atol=1e-12)
    rec0 = oracle.incremental_block_omp(M, y, G, rb, k, prev, 0, True)
    cols = np.concatenate([np.arange(2 * g, 2 * g + 2) for g in prev])
    co, *_ = np.linalg.lstsq(M[:, cols], y, rcond=None)
    assert np.allclose(rec0["coef"], co, atol=1e-12)


def test_orthonormal_dictionary_gives_the_best_support_within_the_budget():
    """With orthonormal atoms the exchange is exactly optimal: brute force over every support that
    shares at least k - swaps units with the previous one."""
    rng = np.random.default_rng(14)
    m, G, k = 16, 12, 4
    for trial in range(6):
        Q, _ = np.linalg.qr(rng.standard_normal((m, G)))
        y = rng.standard_normal(m)
        prev = [int(g) for g in rng.choice(G, size=k, replace=False)]
        for swaps in (1, 2, 3):
            best, best_set = np.inf, None
            for T in itertools.combinations(range(G), k):
                if len(set(T) & set(prev)) < k - swaps:
                    continue
                co = Q[:, T].T @ y
                res = np.linalg.norm(y - Q[:, T] @ co)
                if res < best - 1e-13:
                    best, best_set = res, T
            rec = oracle.incremental_block_omp(Q, y, G, 1, k, prev, swaps, True)
            assert tuple(rec["support"]) == best_set
            assert rec["resid_norm"] == pytest.approx(best, abs=1e-12)
            # closed form: the k - swaps strongest previous units, then the strongest of all the rest
            c = np.abs(Q.T @ y)
            keep = sorted(prev, key=lambda g: -c[g])[:k - swaps]
            rest = sorted((g for g in range(G) if g not in keep), key=lambda g: -c[g])[:swaps]
            assert sorted(keep + rest) == list(rec["support"])


def test_incoherent_dictionary_against_brute_force_within_the_budget():
    rng = np.random.default_rng(15)
    G, m, k, swaps = 12, 40, 4, 2
    hits = 0
    for trial in range(12):
        M, S, alpha = _planted(rng, G, m, k, 2.0, 3.0)
        y = M @ alpha + 1e-3 * rng.standard_normal(m)
        prev = _drift(rng, S, G, swaps)                   # the previous support is `swaps` exchanges away
        best, best_set = np.inf, None
        for T in itertools.combinations(range(G), k):
            if len(set(T) & set(prev.tolist())) < k - swaps:
                continue
            co, *_ = np.linalg.lstsq(M[:, T], y, rcond=None)
            res = np.linalg.norm(y - M[:, T] @ co)
            if res < best:
                best, best_set = res, T
        rec = oracle.incremental_block_omp(M, y, G, 1, k, prev, swaps, True)
        assert best_set == tuple(S)                        # the planted support is the constrained optimum
        hits += tuple(rec["support"]) == best_set
        if tuple(rec["support"]) == best_set:
            assert rec["resid_norm"] == pytest.approx(best, rel=1e-9)
    assert hits >= 11


def test_regularised_refit_closed_form_and_limits():
    rng = np.random.default_rng(16)
    G, m, k = 20, 24, 5
    M = rng.standard_normal((m, G)) / np.sqrt(m)
    y = rng.standard_normal(m)
    prev = [4, 17, 2, 11, 8]
    ap = rng.standard_normal(k)
    A = M[:, prev]
    for gamma in (0.0, 0.3, 10.0):
        rec = oracle.incremental_block_omp(M, y, G, 1, k, prev, 1, True, prev_coef=ap, gamma=gamma)
        want = np.linalg.solve(A.T @ A + gamma * np.eye(k), A.T @ y + gamma * ap)
        assert np.allclose(rec["coef_step1"], want, atol=1e-11)
    # gamma -> infinity: the refit is the previous coefficient vector, so the unit with the least
    # previous energy leaves, whatever y says
    rec = oracle.incremental_block_omp(M, y, G, 1, k, prev, 1, True, prev_coef=ap, gamma=1e12)
    assert np.allclose(rec["coef_step1"], ap, atol=1e-8)
    norms = np.linalg.norm(M, axis=0)
    weakest = prev[int(np.argmin((ap * norms[prev]) ** 2))]
    assert rec["dropped"] == [weakest]
    # without previous coefficients gamma has nothing to pull towards
    a = oracle.incremental_block_omp(M, y, G, 1, k, prev, 2, True, prev_coef=None, gamma=5.0)
    b = oracle.incremental_block_omp(M, y, G, 1, k, prev, 2, True)
    assert list(a["support"]) == list(b["support"]) and np.allclose(a["coef"], b["coef"])


def test_equal_energies_drop_the_larger_index_and_keep_an_exact_support():
    # two identical-energy units: orthonormal atoms, equal |coefficients|
    Q = np.eye(8)[:, :6]
    y = np.array([1.0, 1.0, 3.0, 0.0, 0.0, 0.5, 0.0, 0.0])
    rec = oracle.incremental_block_omp(Q, y, 6, 1, 3, [1, 0, 2], 1, True)
    assert rec["dropped"] == [1]                     # units 0 and 1 tie; the larger index goes first
    assert rec["added"] == [1]                       # ... and comes straight back: it is the best candidate
    assert list(rec["support"]) == [0, 1, 2]
    # previous support already exact and noiseless: any budget returns it unchanged
    rng = np.random.default_rng(17)
    M, S, alpha = _planted(rng, 32, 28, 5)
    y = M @ alpha
    for swaps in (0, 1, 3, 5):
        rec = oracle.incremental_block_omp(M, y, 32, 1, 5, S[::-1], swaps, True)
        assert list(rec["support"]) == list(S)
        assert np.allclose(rec["coef"], alpha[S], atol=1e-9) and rec["resid_norm"] < 1e-10


def test_planted_drift_is_tracked_over_a_token_sequence():
    rng = np.random.default_rng(18)
    G, m, k, swaps = 64, 48, 8, 2
    M = rng.standard_normal((m, G)) / np.sqrt(m)
    S = np.sort(rng.choice(G, size=k, replace=False))
    prev = S.copy()
    for step in range(8):
        S = _drift(rng, S, G, swaps)
        assert oracle.support_drift(S, prev) == pytest.approx(2 * swaps / (k + swaps)) or step > 0
        alpha = np.zeros(G)
        alpha[S] = rng.choice([-1.0, 1.0], size=k) * rng.uniform(1.0, 2.0, size=k)
        y = M @ alpha + 0.01 * rng.standard_normal(m)
        rec = oracle.incremental_block_omp(M, y, G, 1, k, prev, swaps, True)
        assert list(rec["support"]) == list(S)
        assert sorted(rec["added"]) == sorted(set(S.tolist()) - set(prev.tolist()))
        prev = rec["support"]


def test_incremental_recovery_needs_fewer_measurements_than_recovery_from_scratch():
    """Sec. 10, incremental proposition: with the previous support known and a drift of a few
    units, a measurement budget at which recovery from scratch almost always fails identifies the
    new support (the fit on the inherited units still needs m > k; the changed part costs about
    Delta log(eG/Delta) = 4 log(32 e) ~ 18 on top, against k log(eG/k) ~ 49 times a constant)."""
    rng = np.random.default_rng(19)
    G, k, swaps, m = 128, 16, 2, 52
    ok_inc = ok_scratch = 0
    trials = 40
    for trial in range(trials):
        M, S, alpha = _planted(rng, G, m, k, 1.0, 2.0)
        prev = _drift(rng, S, G, swaps)
        y = M @ alpha
        ok_inc += list(oracle.incremental_block_omp(M, y, G, 1, k, prev, swaps, True)["support"]) == list(S)
        ok_scratch += list(oracle.block_omp(M, y, G, 1, k, True)["support"]) == list(S)
    assert ok_inc >= 0.8 * trials              # measured 0.925
    assert ok_scratch <= 0.3 * trials          # measured 0.05


def test_invalid_inputs_are_rejected():
    M = np.eye(8)[:, :6]
    y = np.ones(8)
    with pytest.raises(ValueError):
        oracle.incremental_block_omp(M, y, 6, 1, 3, [0, 1, 1], 1, True)       # repeated unit
    with pytest.raises(ValueError):
        oracle.incremental_block_omp(M, y, 6, 1, 3, [0, 1, 6], 1, True)       # out of range
    with pytest.raises(ValueError):
        oracle.incremental_block_omp(M, y, 6, 1, 3, [0, 1, 2], 4, True)       # budget above k
    with pytest.raises(ValueError):
        oracle.incremental_block_omp(M, y, 6, 1, 3, [0, 1, 2], 1, True, prev_coef=np.zeros(3), gamma=-1.0)
