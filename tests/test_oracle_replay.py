"""Pins for the tie-tolerant replay of the three solvers (CPU only).

A recovered support is a set, and near ties have several correct answers.  The GPU tests accept a
support that differs from the oracle's only if the oracle, told to prefer that support's units within a
small relative slack, reproduces it.  These tests fix what that check accepts and rejects:
 * without a preference, and with the solver's own answer as the preference, nothing changes;
 * a wrong support (the first k units, a support with one unit exchanged) is not reproduced on
   well-separated instances, so a kernel that returned it would fail;
 * at an exact tie (two identical atoms) either choice is accepted, and only at a tie."""
import numpy as np
import pytest
import oracle
from paper_2604_14156_amd import workloads as wl

SLACK = 1e-3


def _planted(rng, G, m, k, noise=0.01):
    M = rng.standard_normal((m, G)) / np.sqrt(m)
    S = np.sort(rng.choice(G, size=k, replace=False))
    alpha = np.zeros(G)
    alpha[S] = rng.uniform(1.0, 2.0, size=k) * rng.choice([-1.0, 1.0], size=k)
    return M, M @ alpha + noise * rng.standard_normal(m), S


def _solvers(M, y, G, k, prev):
    return {
        "omp": lambda **kw: oracle.block_omp(M, y, G, 1, k, True, **kw),
        "iht": lambda **kw: oracle.block_iht(M, y, G, 1, k, 6, True, **kw),
        "inc": lambda **kw: oracle.incremental_block_omp(M, y, G, 1, k, prev, 2, True, **kw),
    }


@pytest.mark.parametrize("name", ["omp", "iht", "inc"])
def test_own_answer_as_preference_changes_nothing(name):
    rng = np.random.default_rng(11)
    for _ in range(5):
        G, m, k = 40, 30, 5
        M, y, S = _planted(rng, G, m, k)
        prev = list(S[:-2]) + [int(g) for g in np.setdiff1d(np.arange(G), S)[:2]]      # two units drifted
        f = _solvers(M, y, G, k, prev)[name]
        plain = f()
        again = f(prefer=plain["support"], slack=SLACK)
        assert list(again["support"]) == list(plain["support"])
        assert again["resid_norm"] == plain["resid_norm"]
        none = f(prefer=[], slack=SLACK)
        assert list(none["support"]) == list(plain["support"])


@pytest.mark.parametrize("name", ["omp", "iht", "inc"])
def test_wrong_supports_are_not_reproduced(name):
    rng = np.random.default_rng(12)
    rejected_first_k = rejected_swapped = 0
    for _ in range(6):
        G, m, k = 40, 30, 5
        M, y, S = _planted(rng, G, m, k)
        prev = list(S[:-2]) + [int(g) for g in np.setdiff1d(np.arange(G), S)[:2]]
        f = _solvers(M, y, G, k, prev)[name]
        plain = f()
        first_k = list(range(k))
        if first_k != list(plain["support"]):
            rejected_first_k += list(f(prefer=first_k, slack=SLACK)["support"]) != first_k
        swapped = list(plain["support"])
        swapped[0] = int(np.setdiff1d(np.arange(G), plain["support"])[-1])
        swapped.sort()
        rejected_swapped += list(f(prefer=swapped, slack=SLACK)["support"]) != swapped
    assert rejected_first_k == 6 and rejected_swapped == 6


def test_exact_tie_accepts_either_unit_and_nothing_else():
    rng = np.random.default_rng(13)
    G, m, k = 12, 20, 3
    M = rng.standard_normal((m, G)) / np.sqrt(m)
    M[:, 9] = M[:, 2]                                   # units 2 and 9 are the same atom
    alpha = np.zeros(G)
    alpha[[2, 5, 7]] = [2.0, -1.5, 1.0]
    y = M @ alpha
    # one round: after unit 2 (or 9) is in, the other has zero score, so k = 1 isolates the tie
    plain = oracle.block_omp(M, y - M[:, [5, 7]] @ alpha[[5, 7]], G, 1, 1, True)
    assert list(plain["support"]) == [2]                # ties -> smaller index
    other = oracle.block_omp(M, y - M[:, [5, 7]] @ alpha[[5, 7]], G, 1, 1, True, prefer=[9], slack=SLACK)
    assert list(other["support"]) == [9]
    wrong = oracle.block_omp(M, y - M[:, [5, 7]] @ alpha[[5, 7]], G, 1, 1, True, prefer=[4], slack=SLACK)
    assert list(wrong["support"]) == [2]
    # hard thresholding, one iteration: the cut falls between the tied pair when k = 1
    iht = oracle.block_iht(M, 2.0 * M[:, 2], G, 1, 1, 1, True, prefer=[9], slack=SLACK)
    assert list(iht["support"]) == [9]
    assert list(oracle.block_iht(M, 2.0 * M[:, 2], G, 1, 1, 1, True)["support"]) == [2]


def test_slack_bounds_what_a_preference_can_change():
    """A preferred unit wins only when its score is within 1/(1+slack) of the best."""
    m = 8
    e = np.eye(m)
    M = e[:, :4].copy()
    y = 1.0 * e[:, 0] + 0.9995 * e[:, 1] + 0.99 * e[:, 2]
    # scores are the squares: 1, 0.9990, 0.9801
    assert list(oracle.block_omp(M, y, 4, 1, 1, True)["support"]) == [0]
    assert list(oracle.block_omp(M, y, 4, 1, 1, True, prefer=[1], slack=2e-3)["support"]) == [1]
    assert list(oracle.block_omp(M, y, 4, 1, 1, True, prefer=[1], slack=5e-4)["support"]) == [0]
    assert list(oracle.block_omp(M, y, 4, 1, 1, True, prefer=[2], slack=2e-3)["support"]) == [0]


def test_decode_shaped_near_tie_is_accepted_both_ways_and_only_within_the_slack():
    """A decode-shaped instance (reduced) whose smallest selection margin is 1.4e-3 and where taking the
    runner-up at that round ends with another support (mostly a near tie only changes the order of
    selection, not the set).  The replay accepts that support with a slack above the gap, rejects it with
    a slack below the gap, and rejects an arbitrary exchange."""
    c = wl.scaled(wl.CFG2, G=86, k=20, m=128)
    seed = 2602
    rng = wl.rng_for(seed)
    pi, psi = wl.make_profiles(rng, c.G, c.b)
    z, S = wl.plant_usage(rng, pi, c.k, 1, c.amp, c.bg)
    M = oracle.effective_matrix(c.ens, seed, 0, c.m, c.G * c.b, c.G, c.b, 1, psi)
    y = oracle.sketch(c.ens, seed, 0, c.m, z[0])
    rec = oracle.block_omp(M, y, c.G, 1, c.k, True)
    assert 1e-3 < rec["margin"] < 2e-3
    alts = []
    for u in range(c.G):
        alt = oracle.block_omp(M, y, c.G, 1, c.k, True, prefer=[u], slack=3e-3)
        if list(alt["support"]) != list(rec["support"]):
            alts.append(alt["support"])
    assert len(alts) >= 1                               # the other way round the near tie
    for alt in alts:
        assert list(oracle.block_omp(M, y, c.G, 1, c.k, True, prefer=alt, slack=3e-3)["support"]) == list(alt)
        assert list(oracle.block_omp(M, y, c.G, 1, c.k, True, prefer=alt, slack=1e-4)["support"]) != list(alt)
    bad = list(rec["support"])
    bad[3] = int(np.setdiff1d(np.arange(c.G), rec["support"])[0])
    bad.sort()
    assert list(oracle.block_omp(M, y, c.G, 1, c.k, True, prefer=bad, slack=3e-3)["support"]) != bad
