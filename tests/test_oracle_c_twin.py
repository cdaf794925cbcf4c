"""Pins for the plain C twin of the decode-step oracle (CPU only): the generator against its published
known-answer vectors, every other function against the NumPy oracle (which carries the pins to the paper
and the mathematics) and, where one exists, against a library routine."""
import os
import numpy as np
import pytest
import oracle
from oracle import c_twin, GAUSS, RADEMACHER
from paper_2604_14156_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_generator_known_answers_and_random_counters():
    for l in open(GOLDEN):
        if l.strip() and not l.startswith("#"):
            v = [int(t, 16) for t in l.split()]
            assert list(c_twin.philox4x32_10(*v[:6])) == v[6:]
    rng = np.random.default_rng(5)
    for _ in range(50):
        v = [int(x) for x in rng.integers(0, 2**32, size=6)]
        assert list(c_twin.philox4x32_10(*v)) == [int(o) for o in oracle.philox4x32_10(*v)]


@pytest.mark.parametrize("ens", [GAUSS, RADEMACHER])
def test_operator_entries_sketch_and_effective_matrix(ens):
    seed, stream, m, n = 0x1234567890AB, 7, 19, 300
    phi = oracle.phi_matrix(ens, seed, stream, m, n) * np.sqrt(m)
    for (i, c) in ((0, 0), (3, 127), (3, 128), (18, 299), (7, 130), (11, 5)):
        assert abs(c_twin.phi_entry(ens, seed, stream, i, c) - phi[i, c]) <= 1e-13 * max(1.0, abs(phi[i, c]))
    rng = np.random.default_rng(2)
    z = rng.standard_normal((5, n))
    want = oracle.sketch(ens, seed, stream, m, z)
    got = c_twin.sketch(ens, seed, stream, m, z)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    assert np.allclose(c_twin.sketch(ens, seed, stream, m, z[2]), want[2], rtol=1e-12, atol=1e-12)
    G, b = 20, 15
    psi = rng.standard_normal((G, b, 1))
    M = oracle.effective_matrix(ens, seed, stream, m, G * b, G, b, 1, psi)
    assert np.allclose(c_twin.effective_matrix(ens, seed, stream, m, G * b, G, b, 1, psi), M, rtol=1e-12, atol=1e-13)
    Mi = oracle.effective_matrix(ens, seed, stream, m, 40, 40, 1, 1, None)
    assert np.allclose(c_twin.effective_matrix(ens, seed, stream, m, 40, 40, 1, 1, None), Mi, rtol=1e-12, atol=1e-13)
    with pytest.raises(ValueError):
        c_twin.effective_matrix(ens, seed, stream, m, 40, 10, 4, 4, None)


@pytest.mark.parametrize("normalised", [True, False])
def test_block_omp_equals_the_numpy_oracle_and_library_least_squares(normalised):
    rng = np.random.default_rng(11)
    m, G, k, B = 48, 30, 7, 6
    M = rng.standard_normal((m, G)) * (1.0 + rng.random(G))          # unequal column norms
    Y = np.empty((B, m))
    for t in range(B):
        S = rng.permutation(G)[:k]
        Y[t] = M[:, S] @ rng.laplace(size=k) + 0.05 * rng.standard_normal(m)
    sup, coef, res, mar = c_twin.block_omp(M, Y, G, k, normalised)
    for t in range(B):
        rec = oracle.block_omp(M, Y[t], G, 1, k, normalised)
        assert list(sup[t]) == list(rec["support"])
        assert np.allclose(coef[t], rec["coef"], rtol=1e-9, atol=1e-11)
        assert abs(res[t] - rec["resid_norm"]) <= 1e-10 * np.linalg.norm(Y[t])
        assert abs(mar[t] - rec["margin"]) <= 1e-9
        ls, *_ = np.linalg.lstsq(M[:, sup[t]], Y[t], rcond=None)
        assert np.allclose(coef[t], ls, rtol=1e-9, atol=1e-11)
    one = c_twin.block_omp(M, Y[3], G, k, normalised)
    assert list(one[0]) == list(sup[3])
    # exact recovery without noise (more rows than the incoherence bound needs), ties -> smaller index
    Q = np.linalg.qr(rng.standard_normal((m, G)))[0]
    y = Q[:, [4, 9]] @ np.array([1.0, 1.0])
    s2 = c_twin.block_omp(Q, y, G, 2, normalised)
    assert list(s2[0]) == [4, 9] and s2[2] <= 1e-12
    with pytest.raises(ValueError):
        c_twin.block_omp(M, Y, G, m, normalised)


def test_block_ffn_and_head_attention_equal_the_numpy_oracle():
    rng = wl.rng_for(77)
    G, b, d, k, T = 9, 24, 40, 4, 5
    Wg, Wu, Wd = wl.make_ffn_weights(rng, G, b, d, 0.2, "f32")
    x = wl.make_tokens(rng, T, d, "f32")
    sup = wl.random_supports(rng, G, k, T)
    assert np.allclose(c_twin.block_ffn(Wg, Wu, Wd, x, sup), oracle.block_ffn(Wg, Wu, Wd, x, sup), rtol=1e-12, atol=1e-13)
    assert np.allclose(c_twin.block_ffn(Wg, Wu, Wd, x, sup[0]), oracle.block_ffn(Wg, Wu, Wd, x, sup[0]), rtol=1e-12, atol=1e-13)
    B, H, L, dh, kh = 3, 6, 37, 16, 2
    q = rng.standard_normal((B, H, dh))
    K = rng.standard_normal((B, H, L, dh))
    V = rng.standard_normal((B, H, L, dh))
    heads = np.stack([np.sort(rng.permutation(H)[:kh]) for _ in range(B)]).astype(np.int32)
    got, want = c_twin.head_attn(q, K, V, heads), oracle.head_attn(q, K, V, heads)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-14)
    assert np.all(got[0, [h for h in range(H) if h not in heads[0]]] == 0.0)


def test_direct_pins_brute_force_masked_dense_and_full_softmax():
    """Pins that do not pass through the NumPy oracle: the best support by exhaustive search (orthonormal
    columns, where the greedy choice is the optimum), the masked dense SwiGLU identity (Sec. 3), full
    softmax attention when every head is kept, and the explicit matrix of the operator entries."""
    import itertools
    rng = np.random.default_rng(23)
    m, G, k = 14, 9, 3
    Q = np.linalg.qr(rng.standard_normal((m, G)))[0]
    y = Q @ (rng.standard_normal(G) * (rng.random(G) > 0.4)) + 0.01 * rng.standard_normal(m)
    best, best_r = None, np.inf
    for S in itertools.combinations(range(G), k):
        a, *_ = np.linalg.lstsq(Q[:, S], y, rcond=None)
        r = np.linalg.norm(y - Q[:, S] @ a)
        if r < best_r:
            best, best_r = S, r
    sup, coef, res, _ = c_twin.block_omp(Q, y, G, k, True)
    assert tuple(sup) == best and abs(res - best_r) <= 1e-12

    Gf, b, d, T, kf = 6, 8, 12, 4, 2
    Wg, Wu = (rng.standard_normal((Gf, b, d)) * 0.3 for _ in range(2))
    Wd = rng.standard_normal((Gf, d, b)) * 0.3                        # a block's slice of the down matrix, [d, b]
    x = rng.standard_normal((T, d))
    S = np.stack([np.sort(rng.permutation(Gf)[:kf]) for _ in range(T)]).astype(np.int32)
    g, u = x @ Wg.reshape(Gf * b, d).T, x @ Wu.reshape(Gf * b, d).T
    mask = np.zeros((T, Gf, b))
    for t in range(T):
        mask[t, S[t]] = 1.0
    hid = (g / (1.0 + np.exp(-g))) * u * mask.reshape(T, Gf * b)
    assert np.allclose(c_twin.block_ffn(Wg, Wu, Wd, x, S), hid @ Wd.transpose(0, 2, 1).reshape(Gf * b, d), rtol=1e-12, atol=1e-13)

    B, H, L, dh = 2, 3, 11, 8
    q, K, V = rng.standard_normal((B, H, dh)), rng.standard_normal((B, H, L, dh)), rng.standard_normal((B, H, L, dh))
    s = np.einsum("bhd,bhld->bhl", q, K) / np.sqrt(dh)
    p = np.exp(s - s.max(-1, keepdims=True))
    full = np.einsum("bhl,bhld->bhd", p / p.sum(-1, keepdims=True), V)
    assert np.allclose(c_twin.head_attn(q, K, V, np.tile(np.arange(H, dtype=np.int32), (B, 1))), full, rtol=1e-12, atol=1e-14)

    seed, stream, mm, n = 99, 2, 6, 10
    Phi = np.array([[c_twin.phi_entry(RADEMACHER, seed, stream, i, c) for c in range(n)] for i in range(mm)])
    assert set(np.unique(Phi)) <= {-1.0, 1.0}
    z = rng.standard_normal(n)
    assert np.allclose(c_twin.sketch(RADEMACHER, seed, stream, mm, z), Phi @ z / np.sqrt(mm), rtol=1e-13, atol=1e-14)
