"""GPU parity: coupled joint selection (pooled sketch of the retained tokens) against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_14156_amd import binding, workloads as wl
from gpu_util import dev_f32, host, rel_err, assert_greedy_support

pytestmark = pytest.mark.gpu

MARGIN = 1e-3
RES_TOL = 1e-5


def _token_sets_agree(tokens, otok, p, k_tok, yt):
    """Tokens identical except for scores within rounding distance of the cut."""
    srt = np.sort(p)[::-1]
    tol = 1e-5 * np.linalg.norm(yt)
    if k_tok == p.size:
        return list(tokens) == list(otok), True
    cut = 0.5 * (srt[k_tok - 1] + srt[k_tok])
    sure_in = set(np.nonzero(p > cut + tol)[0].tolist())
    sure_out = set(np.nonzero(p < cut - tol)[0].tolist())
    got = set(tokens.tolist())
    assert sure_in <= got and not (got & sure_out)
    clear = srt[k_tok - 1] - srt[k_tok] > 2 * tol
    return (list(tokens) == list(otok)) or not clear, clear


@pytest.mark.parametrize("n_tok,m_tok,k_tok,m", [(160, 128, 40, 48), (300, 64, 300, 40), (131, 32, 1, 33), (1000, 128, 129, 64)])
def test_coupled_selection_small(cs, n_tok, m_tok, k_tok, m):
    seed = 6100 + n_tok
    rng = wl.rng_for(seed)
    c = wl.scaled(wl.CFG2, G=24, k=4, m=m, d=64)
    sal, mask = wl.plant_saliency(rng, n_tok, 0.25)
    pi, psi = wl.make_profiles(rng, c.G, c.b)
    S_star = np.sort(rng.choice(c.G, size=c.k, replace=False))
    z = wl.plant_token_usage(rng, pi, S_star, mask, c.k, c.amp, c.bg)
    tok_op = binding.make_op(wl.RADEMACHER, seed, 9, m_tok, n_tok)
    ch_op = binding.make_op(c.ens, seed, 0, c.m, c.n)
    psi_dev = dev_f32(psi)
    dct = binding.make_dict(psi_dev, c.G, c.b, 1)
    y_tok = oracle.sketch(wl.RADEMACHER, seed, 9, m_tok, sal).astype(np.float32)
    Y = oracle.sketch(c.ens, seed, 0, c.m, z).astype(np.float32)
    tokens, support, ybar, resid, margin = cs.cs_joint_select_coupled(tok_op, dev_f32(y_tok), k_tok, ch_op, dct, dev_f32(Y), c.k)
    tokens, support, ybar = host(tokens), host(support), host(ybar)
    M = oracle.effective_matrix(c.ens, seed, 0, c.m, c.n, c.G, c.b, 1, psi)
    otok, oybar, rec, p = oracle.joint_select_coupled((wl.RADEMACHER, seed, 9, m_tok, n_tok), y_tok, k_tok,
                                                      M, Y, c.G, 1, c.k, True)
    assert tokens.shape == (k_tok,) and (k_tok == 1 or np.all(np.diff(tokens) > 0))
    same, clear = _token_sets_agree(tokens, otok, p, k_tok, y_tok)
    assert same
    # the pooled sketch of the tokens the GPU kept, summed in fp64, is what the GPU pooled in fp32
    own = Y[tokens].astype(np.float64).mean(axis=0)
    assert rel_err(ybar, own) <= 1e-5
    if list(tokens) == list(otok):
        assert rel_err(ybar, oybar) <= 1e-5
        if assert_greedy_support(M, oybar, c.G, 1, c.k, True, support, rec):
            assert abs(host(resid)[0] - rec["resid_norm"]) <= RES_TOL * np.linalg.norm(oybar) + 1e-5 * np.linalg.norm(oybar)


def test_coupled_selection_prompt_shape_full_size(cs):
    """8192 prompt tokens, 2048 kept, per-token channel sketches produced by the library's own
    sketch call; the oracle pools the usage instead and sketches once (linearity)."""
    t = wl.CFG5_TOK
    c = wl.CFG2
    seed = 6200
    rng = wl.rng_for(seed)
    n_tok, k_tok = t["n_tok"], t["k_tok"]
    sal, mask = wl.plant_saliency(rng, n_tok, t["p_active"])
    pi, psi = wl.make_profiles(rng, c.G, c.b)
    S_star = np.sort(rng.choice(c.G, size=c.k, replace=False))
    # usage on the device: salient tokens share S*, the others draw their own k units
    gen = torch.Generator(device="cuda:0").manual_seed(seed)
    pi_d = dev_f32(pi)
    perm = torch.rand((n_tok, c.G), generator=gen, device="cuda:0").argsort(dim=1)[:, :c.k]
    star = torch.from_numpy(S_star.astype(np.int64)).to("cuda:0")
    mask_d = torch.from_numpy(mask).to("cuda:0")
    units = torch.where(mask_d[:, None], star[None, :].expand(n_tok, c.k), perm)
    amp = torch.zeros((n_tok, c.G), device="cuda:0")
    mag = 0.5 + torch.rand((n_tok, c.k), generator=gen, device="cuda:0")          # one sign: the mean does not cancel
    amp.scatter_(1, units, mag)
    tok_op = binding.make_op(t["ens"], seed, 9, t["m_tok"], n_tok)
    ch_op = binding.make_op(c.ens, seed, 0, c.m, c.n)
    psi_dev = dev_f32(psi)
    dct = binding.make_dict(psi_dev, c.G, c.b, 1)
    Y = torch.empty((n_tok, c.m), device="cuda:0")
    for i0 in range(0, n_tok, 1024):                                              # 45 MB of usage at a time
        z = (amp[i0:i0 + 1024, :, None] * pi_d[None]).reshape(-1, c.n).contiguous()
        cs.cs_sketch(ch_op, z, Y[i0:i0 + 1024])
    y_tok = cs.cs_sketch(tok_op, dev_f32(sal[None, :]))[0]
    tokens, support, ybar, resid, margin = cs.cs_joint_select_coupled(tok_op, y_tok, k_tok, ch_op, dct, Y, c.k)
    tokens, support, ybar = host(tokens), host(support), host(ybar)
    yt = host(y_tok)
    p = oracle.token_proxy(t["ens"], seed, 9, t["m_tok"], n_tok, yt)
    otok = oracle.top_k_indices(p, k_tok)
    same, clear = _token_sets_agree(tokens, otok, p, k_tok, yt)
    assert same
    # oracle side: pooled usage of the tokens the GPU kept -> one sketch -> block-OMP
    idx = torch.from_numpy(tokens.astype(np.int64)).to("cuda:0")
    abar = host(amp[idx].double().mean(dim=0))                                    # [G] mean magnitudes
    zbar = (abar[:, None] * pi.astype(np.float64)).reshape(-1)
    want = oracle.sketch(c.ens, seed, 0, c.m, zbar)
    assert rel_err(ybar, want) <= 1e-5
    M = oracle.effective_matrix(c.ens, seed, 0, c.m, c.n, c.G, c.b, 1, psi)
    rec = oracle.block_omp(M, want, c.G, 1, c.k, True)
    assert_greedy_support(M, want, c.G, 1, c.k, True, support, rec)
