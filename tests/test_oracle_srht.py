"""Pins for the oracle's subsampled randomised Hadamard operator (CPU only).

Sec. 8 names the ensemble; the construction R H D is the textbook one.  The pins tie the
entrywise definition to a library Hadamard matrix, to a textbook fast transform and to the
properties the construction must have; which signs and rows a (seed, stream) pair selects is
this project's own convention.
"""
import numpy as np
import pytest
import scipy.linalg
import oracle
from oracle import SRHT


def _fwht(v):
    """Textbook in-place fast Walsh-Hadamard transform (natural order)."""
    v = np.array(v, dtype=np.float64)
    h = 1
    while h < v.size:
        for i in range(0, v.size, 2 * h):
            a = v[i:i + h].copy()
            b = v[i + h:i + 2 * h].copy()
            v[i:i + h] = a + b
            v[i + h:i + 2 * h] = a - b
        h *= 2
    return v


def test_order_and_row_map_is_a_bijection():
    assert oracle.srht_order(1) == (2, 1) and oracle.srht_order(2) == (2, 1)
    assert oracle.srht_order(64) == (64, 6) and oracle.srht_order(65) == (128, 7)
    assert oracle.srht_order(11008) == (16384, 14)
    for n, seed in ((64, 1), (100, 2), (2, 3), (11008, 4)):
        npad, _ = oracle.srht_order(n)
        r = oracle.srht_rows(seed, 5, np.arange(npad), n)
        assert sorted(r.tolist()) == list(range(npad))
    # different seeds or streams give different row choices
    a = oracle.srht_rows(7, 0, np.arange(16), 1024)
    assert not np.array_equal(a, oracle.srht_rows(8, 0, np.arange(16), 1024))
    assert not np.array_equal(a, oracle.srht_rows(7, 1, np.arange(16), 1024))


@pytest.mark.parametrize("n,m", [(64, 16), (100, 40), (128, 128), (5, 3)])
def test_matrix_is_R_H_D_with_a_library_hadamard(n, m):
    seed, stream = 11, 3
    npad, _ = oracle.srht_order(n)
    phi = oracle.phi_matrix(SRHT, seed, stream, m, n)
    H = scipy.linalg.hadamard(npad).astype(np.float64)          # Sylvester order: H[r, c] = (-1)**popcount(r & c)
    rows = oracle.srht_rows(seed, stream, np.arange(m), n).astype(np.int64)
    d = phi[0] * np.sqrt(m) * H[rows[0], :n]                     # signs recovered from the first row ...
    assert set(np.unique(d).tolist()) <= {-1.0, 1.0}
    want = H[rows][:, :n] * d[None, :] / np.sqrt(m)              # ... must explain every other row
    assert np.array_equal(phi, want)
    # the signs are the Rademacher bits of the documented counter, not a function of the row
    assert abs(d.mean()) < 0.5 or n < 16
    # column slices agree with the full matrix
    assert np.array_equal(oracle.phi_matrix(SRHT, seed, stream, m, n, 3, 2), phi[:, 3:5])


def test_rows_are_orthogonal_and_nested():
    n, m = 256, 64
    phi = oracle.phi_matrix(SRHT, 21, 0, m, n)
    assert np.allclose(phi @ phi.T, (n / m) * np.eye(m), atol=1e-12)
    assert np.allclose(np.linalg.norm(phi, axis=0), 1.0, atol=1e-12)        # unit-norm columns
    half = oracle.phi_matrix(SRHT, 21, 0, m // 2, n)
    assert np.allclose(half * np.sqrt(m // 2), phi[:m // 2] * np.sqrt(m), atol=1e-12)
    with pytest.raises(ValueError):
        oracle.phi_matrix(SRHT, 21, 0, 300, 256)                              # more rows than the transform has


def test_sketch_equals_a_fast_transform_of_the_signed_padded_vector():
    rng = np.random.default_rng(5)
    n, m, seed, stream = 300, 48, 31, 2
    npad, _ = oracle.srht_order(n)
    z = rng.standard_normal(n)
    y = oracle.sketch(SRHT, seed, stream, m, z)
    phi = oracle.phi_matrix(SRHT, seed, stream, m, n)
    assert np.allclose(y, phi @ z, atol=1e-12)
    H = scipy.linalg.hadamard(npad).astype(np.float64)
    rows = oracle.srht_rows(seed, stream, np.arange(m), n).astype(np.int64)
    d = phi[0] * np.sqrt(m) * H[rows[0], :n]
    padded = np.zeros(npad)
    padded[:n] = d * z
    assert np.allclose(y, _fwht(padded)[rows] / np.sqrt(m), atol=1e-10)


def test_norm_is_preserved_in_expectation_and_recovery_works():
    rng = np.random.default_rng(6)
    n, m = 512, 128
    z = rng.standard_normal(n)
    ratios = [np.sum(oracle.sketch(SRHT, s, 0, m, z) ** 2) / np.sum(z ** 2) for s in range(40)]
    assert abs(np.mean(ratios) - 1.0) < 0.1
    # the operator is as good a sensing matrix as the dense ensembles: planted supports come back
    G, b, k = 64, 8, 4
    hits = 0
    for trial in range(5):
        pi = rng.standard_normal((G, b))
        psi = (pi / np.linalg.norm(pi, axis=1, keepdims=True)).reshape(G, b, 1)
        S = np.sort(rng.choice(G, size=k, replace=False))
        u = np.zeros(G * b)
        for g in S:
            u[g * b:(g + 1) * b] = rng.choice([-1.0, 1.0]) * rng.uniform(1, 2) * pi[g]
        M = oracle.effective_matrix(SRHT, 50 + trial, 1, 48, G * b, G, b, 1, psi)
        y = oracle.sketch(SRHT, 50 + trial, 1, 48, u)
        hits += list(oracle.block_omp(M, y, G, 1, k, True)["support"]) == list(S)
    assert hits >= 4
