"""Pins for the oracle's generator, operator and sketch (CPU only)."""
import math
import os
import numpy as np
import oracle
from oracle import GAUSS, RADEMACHER

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 2
    for r in rows:
        v = [int(t, 16) for t in r]
        out = oracle.philox4x32_10(*v[:6])
        assert [int(o) for o in out] == v[6:]


def test_philox_scalar_reimplementation_matches_vectorised():
    # an independent scalar transcription of the round function (Python ints)
    def scalar(c, k):
        c, k = list(c), list(k)
        for rnd in range(10):
            if rnd:
                k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
            p0, p1 = 0xD2511F53 * c[0], 0xCD9E8D57 * c[2]
            c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
        return c
    rng = np.random.default_rng(1)
    for _ in range(20):
        v = [int(x) for x in rng.integers(0, 2**32, size=6)]
        assert [int(o) for o in oracle.philox4x32_10(*v)] == scalar(v[:4], v[4:])


def test_rademacher_entries_are_signs_with_unit_columns():
    phi = oracle.phi_matrix(RADEMACHER, 7, 3, 64, 1000)
    assert set(np.unique(phi * 8.0)) == {-1.0, 1.0}
    assert np.allclose((phi ** 2).sum(axis=0), 1.0, atol=1e-14)
    # balanced signs and weak column coherence (a stuck bit or a reused word would break these)
    assert abs(phi.sum()) * 8.0 < 5 * math.sqrt(phi.size)
    gram = phi.T @ phi
    np.fill_diagonal(gram, 0.0)
    assert np.abs(gram).max() < 0.75


def test_rademacher_bit_convention():
    # column c takes bit (c mod 32) of word ((c mod 128) // 32) of call c // 128
    seed, stream, row = 0x1234567812345678, 5, 9
    for col in (0, 31, 32, 127, 128, 300):
        w = oracle.philox4x32_10(col // 128, row, stream, RADEMACHER, seed & 0xFFFFFFFF, seed >> 32)
        bit = (int(w[(col % 128) // 32]) >> (col % 32)) & 1
        e = oracle.phi_entries(RADEMACHER, seed, stream, row, col)
        assert float(e) == (1.0 if bit == 0 else -1.0)


def test_gaussian_moments_and_pairing():
    e = oracle.phi_entries(GAUSS, 11, 0, np.arange(400)[:, None], np.arange(1000)[None, :])
    n = e.size
    assert abs(e.mean()) < 5 / math.sqrt(n)
    assert abs(e.var() - 1.0) < 5 * math.sqrt(2.0 / n)
    assert abs((e ** 4).mean() - 3.0) < 5 * math.sqrt(96.0 / n)
    # Box-Muller pairing: an even/odd column pair shares its radius
    w = oracle.philox4x32_10(0, 3, 0, GAUSS, 11, 0)
    rad2 = -2.0 * math.log((int(w[0]) + 1) / 2.0**32)
    pair = oracle.phi_entries(GAUSS, 11, 0, 3, np.array([0, 1]))
    assert abs(pair[0] ** 2 + pair[1] ** 2 - rad2) < 1e-12
    ang = 2.0 * math.pi * (int(w[1]) + 1) / 2.0**32
    assert abs(pair[0] - math.sqrt(rad2) * math.cos(ang)) < 1e-12
    # distinct rows / streams / seeds decorrelate
    a = oracle.phi_entries(GAUSS, 11, 0, 0, np.arange(4000))
    for other in (oracle.phi_entries(GAUSS, 11, 0, 1, np.arange(4000)),
                  oracle.phi_entries(GAUSS, 11, 1, 0, np.arange(4000)),
                  oracle.phi_entries(GAUSS, 12, 0, 0, np.arange(4000))):
        assert abs(np.corrcoef(a, other)[0, 1]) < 0.08


def test_rows_are_nested_in_m():
    for ens in (GAUSS, RADEMACHER):
        small = oracle.phi_matrix(ens, 5, 2, 16, 200) * math.sqrt(16)
        big = oracle.phi_matrix(ens, 5, 2, 48, 200) * math.sqrt(48)
        assert np.allclose(small, big[:16], atol=1e-13)


def test_sketch_equals_entrywise_definition():
    rng = np.random.default_rng(3)
    for ens in (GAUSS, RADEMACHER):
        m, n = 5, 300
        z = rng.standard_normal(n)
        y = oracle.sketch(ens, 21, 4, m, z, col_chunk=128)
        for i in range(m):
            acc = 0.0
            for j in range(n):
                acc += float(oracle.phi_entries(ens, 21, 4, i, j)) * z[j]
            assert abs(y[i] - acc / math.sqrt(m)) < 1e-12


def test_sketch_linearity_and_batching():
    rng = np.random.default_rng(4)
    z1, z2 = rng.standard_normal((2, 777))
    y1 = oracle.sketch(RADEMACHER, 9, 0, 32, z1)
    y2 = oracle.sketch(RADEMACHER, 9, 0, 32, z2)
    y12 = oracle.sketch(RADEMACHER, 9, 0, 32, 2.5 * z1 + z2)
    assert np.allclose(y12, 2.5 * y1 + y2, atol=1e-12)
    yb = oracle.sketch(RADEMACHER, 9, 0, 32, np.stack([z1, z2]))
    assert np.allclose(yb[0], y1) and np.allclose(yb[1], y2)


def test_sketch_preserves_norm_in_expectation():
    rng = np.random.default_rng(5)
    z = rng.standard_normal(512)
    for ens in (GAUSS, RADEMACHER):
        ratios = [np.sum(oracle.sketch(ens, 100 + s, s, 64, z) ** 2) / np.sum(z ** 2)
                  for s in range(60)]
        # each ratio has variance ~ 2/m; the mean of 60 has std ~ 0.023
        assert abs(np.mean(ratios) - 1.0) < 0.1
