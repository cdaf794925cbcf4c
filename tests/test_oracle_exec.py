"""Pins for the oracle's execution side (FFN, attention, top-k, joint), CPU only."""
import math
import numpy as np
import torch
import oracle
from oracle import RADEMACHER
from paper_2604_14156_amd import workloads as wl


def _small_ffn(seed, G=6, b=8, d=24, T=3):
    rng = wl.rng_for(seed)
    Wg, Wu, Wd = wl.make_ffn_weights(rng, G, b, d, 0.3, "f32")
    x = wl.make_tokens(rng, T, d, "f32")
    return Wg, Wu, Wd, x


def test_ffn_all_blocks_is_dense_swiglu():
    G, b, d, T = 6, 8, 24, 3
    Wg, Wu, Wd, x = _small_ffn(1, G, b, d, T)
    out = oracle.block_ffn(Wg, Wu, Wd, x, np.arange(G))
    # independent dense formulation with library ops (torch CPU, fp64)
    tg = torch.from_numpy(Wg.reshape(G * b, d)).double()
    tu = torch.from_numpy(Wu.reshape(G * b, d)).double()
    # dense down projection [d, d_ff]: column c = g*b + j is Wd[g, :, j]
    td = torch.from_numpy(Wd).double().permute(1, 0, 2).reshape(d, G * b)
    tx = torch.from_numpy(x).double()
    ref = (torch.nn.functional.silu(tx @ tg.T) * (tx @ tu.T)) @ td.T
    assert np.allclose(out, ref.numpy(), rtol=1e-12, atol=1e-12)


def test_ffn_masked_dense_identity_and_additivity():
    G, b, d, T = 6, 8, 24, 3
    Wg, Wu, Wd, x = _small_ffn(2, G, b, d, T)
    S = np.array([1, 4, 5])
    out = oracle.block_ffn(Wg, Wu, Wd, x, S)
    # Sec. 3: reduced execution == dense execution with the other units zeroed
    Wg0, Wu0, Wd0 = Wg.copy(), Wu.copy(), Wd.copy()
    for g in range(G):
        if g not in S:
            Wd0[g] = 0.0
    assert np.allclose(out, oracle.block_ffn(Wg0, Wu0, Wd0, x, np.arange(G)), atol=1e-13)
    # additivity over disjoint supports, and order independence
    a = oracle.block_ffn(Wg, Wu, Wd, x, np.array([1]))
    bb = oracle.block_ffn(Wg, Wu, Wd, x, np.array([4, 5]))
    assert np.allclose(out, a + bb, atol=1e-13)
    assert np.allclose(out, oracle.block_ffn(Wg, Wu, Wd, x, S[::-1]), atol=1e-13)
    # per-token supports: row t uses only its own list
    per = np.array([[0, 1], [2, 3], [4, 5]])
    o = oracle.block_ffn(Wg, Wu, Wd, x, per)
    for t in range(T):
        assert np.allclose(o[t], oracle.block_ffn(Wg, Wu, Wd, x[t:t + 1], per[t])[0], atol=1e-13)


def test_ffn_hand_computed_single_channel():
    # one block, one channel: out = silu(wg.x) * (wu.x) * wd
    Wg = np.array([[[1.0, 2.0]]]); Wu = np.array([[[0.5, -1.0]]]); Wd = np.array([[[3.0], [-2.0]]])
    x = np.array([[1.0, 1.0]])
    gate, up = 3.0, -0.5
    h = gate / (1.0 + math.exp(-gate)) * up
    out = oracle.block_ffn(Wg, Wu, Wd, x, np.array([0]))
    assert np.allclose(out, [[3.0 * h, -2.0 * h]], atol=1e-15)


def test_attention_all_heads_is_softmax_attention():
    rng = wl.rng_for(3)
    B, H, L, dh = 2, 3, 17, 8
    q, K, V = wl.make_kv(rng, B, H, L, dh)
    out = oracle.head_attn(q, K, V, np.tile(np.arange(H), (B, 1)))
    tq, tK, tV = (torch.from_numpy(a).double() for a in (q, K, V))
    ref = torch.softmax(torch.einsum("bhd,bhld->bhl", tq, tK) / math.sqrt(dh), dim=-1)
    ref = torch.einsum("bhl,bhld->bhd", ref, tV)
    assert np.allclose(out, ref.numpy(), atol=1e-12)


def test_attention_pruned_heads_are_zero_and_closed_forms():
    rng = wl.rng_for(4)
    B, H, L, dh = 2, 4, 9, 8
    q, K, V = wl.make_kv(rng, B, H, L, dh)
    heads = np.array([[0, 2], [1, 3]])
    out = oracle.head_attn(q, K, V, heads)
    assert np.all(out[0, 1] == 0) and np.all(out[0, 3] == 0) and np.all(out[1, 0] == 0)
    assert np.abs(out[0, 0]).sum() > 0
    # L = 1: the only value is returned
    o1 = oracle.head_attn(q, K[:, :, :1], V[:, :, :1], heads)
    assert np.allclose(o1[0, 2], V[0, 2, 0], atol=1e-14)
    # identical keys: uniform weights, output = mean of values
    Ku = np.broadcast_to(K[:, :, :1], K.shape)
    ou = oracle.head_attn(q, Ku, V, heads)
    assert np.allclose(ou[1, 3], V[1, 3].astype(np.float64).mean(axis=0), atol=1e-13)
    # a key aligned with a huge query takes all the weight
    qb = q.copy(); qb[0, 0] = 200.0 * K[0, 0, 5]
    ob = oracle.head_attn(qb, K, V, heads)
    assert np.allclose(ob[0, 0], V[0, 0, 5], atol=1e-6)


def test_top_k_matches_full_sort_with_ties():
    rng = np.random.default_rng(5)
    s = rng.integers(-3, 4, size=50).astype(np.float64)          # many ties
    for k in (1, 7, 25, 50):
        got = oracle.top_k_indices(s, k)
        order = np.lexsort((np.arange(50), -s))                  # by -score, then index
        assert list(got) == sorted(order[:k].tolist())
    assert list(oracle.top_k_indices(s, 50)) == list(range(50))
    # signed: a large negative score is not kept
    assert list(oracle.top_k_indices(np.array([-9.0, 1.0, 0.5]), 2)) == [1, 2]
    # permutation equivariance on distinct scores
    s = rng.standard_normal(40)
    perm = rng.permutation(40)
    a = set(oracle.top_k_indices(s, 10).tolist())
    b = set(perm[oracle.top_k_indices(s[perm], 10)].tolist())
    assert a == b


def test_token_proxy_is_backprojection_and_joint_composes():
    rng = wl.rng_for(6)
    n_tok, m_tok, k_tok = 96, 24, 24
    sal, mask = wl.plant_saliency(rng, n_tok, 0.25)
    op = (RADEMACHER, 77, 3, m_tok, n_tok)
    y_tok = oracle.sketch(RADEMACHER, 77, 3, m_tok, sal)
    p = oracle.token_proxy(*op, y_tok)
    # entrywise definition p_j = sum_i Phi_ij y_i
    for j in (0, 31, 95):
        acc = sum(float(oracle.phi_entries(RADEMACHER, 77, 3, i, j)) * y_tok[i] for i in range(m_tok))
        assert abs(p[j] - acc / math.sqrt(m_tok)) < 1e-12
    # with m = n and orthogonal rows the proxy would return the saliency; here it must at least
    # correlate with it (unit-norm columns: E p_j = s_j)
    assert np.corrcoef(p, sal)[0, 1] > 0.3
    G, k = 12, 3
    M = rng.standard_normal((20, G))
    alpha = np.zeros(G); alpha[[2, 5, 7]] = [3.0, -4.0, 5.0]
    tokens, rec, p2 = oracle.joint_select(op, y_tok, k_tok, M, M @ alpha, G, 1, k, True)
    assert np.allclose(p, p2)
    assert list(tokens) == list(oracle.top_k_indices(p, k_tok))
    assert list(rec["support"]) == [2, 5, 7]


def test_coupled_joint_selection_pools_the_kept_tokens_only():
    """Sec. 6: the retained tokens change the measurement the support is recovered from."""
    rng = wl.rng_for(8)
    n_tok, m_tok, k_tok = 160, 128, 40
    c = wl.scaled(wl.CFG2, G=24, k=4, m=48, d=64)
    sal, mask = wl.plant_saliency(rng, n_tok, 0.25)
    pi, psi = wl.make_profiles(rng, c.G, c.b)
    S_star = np.sort(rng.choice(c.G, size=c.k, replace=False))
    # the salient tokens share S* with magnitudes of one sign, so that their mean does not cancel
    z = wl.plant_token_usage(rng, np.abs(pi), S_star, mask, c.k, "unit", 0.0)
    tok_op = (RADEMACHER, 81, 3, m_tok, n_tok)
    y_tok = oracle.sketch(RADEMACHER, 81, 3, m_tok, sal)
    psi_abs = np.abs(pi) / np.linalg.norm(pi, axis=1, keepdims=True)
    M = oracle.effective_matrix(c.ens, 81, 0, c.m, c.n, c.G, c.b, 1, psi_abs.reshape(c.G, c.b, 1))
    Y = oracle.sketch(c.ens, 81, 0, c.m, z)
    tokens, ybar, rec, p = oracle.joint_select_coupled(tok_op, y_tok, k_tok, M, Y, c.G, 1, c.k, True)
    assert list(tokens) == list(oracle.top_k_indices(p, k_tok))
    # linearity: the pooled sketch is the sketch of the pooled usage
    zbar = z[tokens].astype(np.float64).mean(axis=0)
    assert np.allclose(ybar, oracle.sketch(c.ens, 81, 0, c.m, zbar), atol=1e-12)
    assert np.allclose(ybar, Y[tokens].mean(axis=0), atol=1e-12)
    # keeping every token pools the whole prompt
    t_all, ybar_all, rec_all, _ = oracle.joint_select_coupled(tok_op, y_tok, n_tok, M, Y, c.G, 1, c.k, True)
    assert list(t_all) == list(range(n_tok)) and np.allclose(ybar_all, Y.mean(axis=0), atol=1e-12)
    # the kept tokens are mostly the salient ones, which share S*: the coupled recovery finds it ...
    assert mask[tokens].mean() > 0.5          # base rate 0.25
    assert list(rec["support"]) == list(S_star)
    # ... and it is the token selection that does it: over tokens that do not share a support the
    # pooled sketch has no common support to find
    others = np.nonzero(~mask)[0][:k_tok]
    rec_other = oracle.block_omp(M, Y[others].mean(axis=0), c.G, 1, c.k, True)
    assert list(rec_other["support"]) != list(S_star)
