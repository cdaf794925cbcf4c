"""GPU parity: warm-started (incremental) recovery against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_14156_amd import binding, workloads as wl
from gpu_util import dev_f32, dev_i32, host

pytestmark = pytest.mark.gpu

MARGIN = 1e-3          # supports are compared bit-exactly only when the oracle's decisions are this clear
SLACK = 1e-3           # below that: the oracle, preferring the GPU's units within this slack, must reproduce them
RES_TOL = 1e-5


def _check(cs, op, dct, M, Y, G, k, prev, swaps, normalised, prev_coef=None, gamma=0.0, state=None):
    """state: a carried-state buffer -> the call goes through cs_recover_support_inc_carry."""
    if state is None:
        sup, coef, resid, margin = cs.cs_recover_support_inc(
            op, dct, k, dev_f32(Y), dev_i32(prev), swaps,
            prev_coef=None if prev_coef is None else dev_f32(prev_coef), gamma=gamma)
    else:
        sup, coef, resid, margin = cs.cs_recover_support_inc_carry(op, dct, k, dev_f32(Y), dev_i32(prev), swaps, state)
    sup, coef, resid, margin = host(sup), host(coef), host(resid), host(margin)
    _check.last_support = sup
    exact = 0
    for t in range(Y.shape[0]):
        y = Y[t].astype(np.float64)
        rec = oracle.incremental_block_omp(M, y, G, 1, k, prev[t], swaps, normalised,
                                           prev_coef=None if prev_coef is None else prev_coef[t].astype(np.float64),
                                           gamma=gamma)
        s = sup[t]
        assert len(set(s.tolist())) == k and np.all(np.diff(s) > 0) and s.min() >= 0 and s.max() < G, (t, s)
        assert len(set(s.tolist()) & set(prev[t].tolist())) >= k - swaps          # within the drift budget
        ls, *_ = np.linalg.lstsq(M[:, s], y, rcond=None)
        own = np.linalg.norm(y - M[:, s] @ ls)
        ynorm = np.linalg.norm(y)
        assert abs(resid[t] - own) <= RES_TOL * ynorm
        assert np.linalg.norm(coef[t] - ls) <= 1e-4 * max(np.linalg.norm(ls), 1e-30)
        if rec["margin"] > MARGIN and rec["drop_margin"] > MARGIN:
            assert list(s) == list(rec["support"]), (t, rec["margin"], rec["drop_margin"])
            assert abs(resid[t] - rec["resid_norm"]) <= RES_TOL * ynorm
            assert abs(margin[t] - rec["margin"]) <= 1e-3
            exact += 1
        elif list(s) == list(rec["support"]):
            assert abs(resid[t] - rec["resid_norm"]) <= RES_TOL * ynorm      # a near tie resolved as the plain rule does
        else:
            rep = oracle.incremental_block_omp(M, y, G, 1, k, prev[t], swaps, normalised,
                                               prev_coef=None if prev_coef is None else prev_coef[t].astype(np.float64),
                                               gamma=gamma, prefer=s, slack=SLACK)
            assert list(rep["support"]) == list(s), (t, rec["margin"], rec["drop_margin"], sorted(set(s) ^ set(rec["support"])))
            assert abs(resid[t] - rep["resid_norm"]) <= RES_TOL * ynorm
    return exact


def _decode_case(seed, B, true_swaps):
    c = wl.CFG2
    rng = wl.rng_for(seed)
    pi, psi = wl.make_profiles(rng, c.G, c.b)
    _, S_prev = wl.plant_usage(rng, pi, c.k, B, c.amp, c.bg)
    S_now = wl.drift_supports(rng, S_prev, c.G, true_swaps)
    z = wl.plant_usage_on(rng, pi, S_now, c.amp, c.bg)
    op = binding.make_op(c.ens, seed, 4, c.m, c.n)
    psi_dev = dev_f32(psi)
    dct = binding.make_dict(psi_dev, c.G, c.b, 1)
    M = oracle.effective_matrix(c.ens, seed, 4, c.m, c.n, c.G, c.b, 1, psi)
    Y = oracle.sketch(c.ens, seed, 4, c.m, z).astype(np.float32)
    prev = np.stack([rng.permutation(S_prev[t]) for t in range(B)]).astype(np.int32)     # any order
    return c, op, dct, psi_dev, M, Y, prev, S_now, rng


@pytest.mark.parametrize("swaps,true_swaps", [(0, 0), (1, 1), (4, 3), (12, 12), (43, 5)])
def test_incremental_decode_shape(cs, swaps, true_swaps):
    c, op, dct, psi_dev, M, Y, prev, S_now, rng = _decode_case(4100 + swaps, 5, true_swaps)
    cs.cs_plan(op, dct, psi_dev)
    exact = _check(cs, op, dct, M, Y, c.G, c.k, prev, swaps, True)
    assert exact == 5          # every instance of these seeds is compared bit for bit


def test_incremental_literal_entrywise_usage(cs):
    """Usage drawn entry by entry lies outside the dictionary's span; the third instance has a greedy
    margin of 2e-4 and goes through the near-tie replay, the others are compared bit for bit."""
    c = wl.CFG2
    seed = 2100
    rng = wl.rng_for(seed)
    _, psi = wl.make_profiles(rng, c.G, c.b)
    z, S = wl.plant_usage_literal(rng, c.G, c.b, c.k, 4, c.amp, c.bg)
    op = binding.make_op(c.ens, seed, 0, c.m, c.n)
    psi_dev = dev_f32(psi)
    dct = binding.make_dict(psi_dev, c.G, c.b, 1)
    cs.cs_plan(op, dct, psi_dev)
    M = oracle.effective_matrix(c.ens, seed, 0, c.m, c.n, c.G, c.b, 1, psi)
    Y = oracle.sketch(c.ens, seed, 0, c.m, z).astype(np.float32)
    assert _check(cs, op, dct, M, Y, c.G, c.k, S.astype(np.int32), 6, True) == 3


def test_incremental_with_temporal_regulariser(cs):
    c, op, dct, psi_dev, M, Y, prev, S_now, rng = _decode_case(4200, 4, 3)
    cs.cs_plan(op, dct, psi_dev)
    prev_coef = rng.laplace(0.0, 1.0, size=prev.shape).astype(np.float32)
    for gamma in (0.05, 2.0):
        assert _check(cs, op, dct, M, Y, c.G, c.k, prev, 4, True, prev_coef=prev_coef, gamma=gamma) == 4
    # gamma without previous coefficients is the unregularised call
    a = host(cs.cs_recover_support_inc(op, dct, c.k, dev_f32(Y), dev_i32(prev), 4, gamma=3.0)[0])
    b = host(cs.cs_recover_support_inc(op, dct, c.k, dev_f32(Y), dev_i32(prev), 4)[0])
    assert np.array_equal(a, b)


def test_full_budget_equals_recovery_from_scratch_and_in_place_update(cs):
    c, op, dct, psi_dev, M, Y, prev, S_now, rng = _decode_case(4300, 4, 2)
    cs.cs_plan(op, dct, psi_dev)
    y = dev_f32(Y)
    ref = cs.cs_recover_support(op, dct, c.k, y)
    got = cs.cs_recover_support_inc(op, dct, c.k, y, dev_i32(prev), c.k)
    assert np.array_equal(host(got[0]), host(ref[0]))
    assert np.allclose(host(got[2]), host(ref[2]), rtol=0, atol=RES_TOL * np.linalg.norm(Y, axis=1).max())
    # the support buffer may be the previous-support buffer
    buf = dev_i32(prev)
    want = host(cs.cs_recover_support_inc(op, dct, c.k, y, dev_i32(prev), 3)[0])
    cs.cs_recover_support_inc(op, dct, c.k, y, buf, 3, support=buf)
    assert np.array_equal(host(buf), want)


def test_incremental_head_selection_identity_dictionary(cs):
    hs = wl.CFG3_HEADS
    seed = 4400
    rng = wl.rng_for(seed)
    B = 8
    _, S_prev = wl.plant_head_usage(rng, hs, B)
    S_now = wl.drift_supports(rng, S_prev, hs.H, 2)
    u = (hs.bg * rng.standard_normal((B, hs.H)))
    for t in range(B):
        u[t, S_now[t]] += rng.standard_normal(hs.kh)
    op = binding.make_op(hs.ens, seed, 3, hs.m, hs.H)
    dct = binding.make_dict(None, hs.H, 1, 1)
    M = oracle.effective_matrix(hs.ens, seed, 3, hs.m, hs.H, hs.H, 1, 1, None)
    Y = oracle.sketch(hs.ens, seed, 3, hs.m, u.astype(np.float32)).astype(np.float32)
    for swaps in (0, 2, 5):
        assert _check(cs, op, dct, M, Y, hs.H, hs.kh, S_prev.astype(np.int32), swaps, False) == 8


def test_invalid_rows_and_arguments(cs):
    c, op, dct, psi_dev, M, Y, prev, S_now, rng = _decode_case(4500, 3, 2)
    cs.cs_plan(op, dct, psi_dev)
    bad = prev.copy()
    bad[0, 5] = bad[0, 6]              # a repeated unit
    bad[2, 0] = c.G                    # out of range
    sup, coef, resid, margin = cs.cs_recover_support_inc(op, dct, c.k, dev_f32(Y), dev_i32(bad), 2)
    sup, coef, resid, margin = host(sup), host(coef), host(resid), host(margin)
    for t in (0, 2):
        assert np.all(sup[t] == -1) and np.all(coef[t] == 0.0) and np.isnan(resid[t]) and margin[t] == 0.0
    rec = oracle.incremental_block_omp(M, Y[1].astype(np.float64), c.G, 1, c.k, prev[1], 2, True)
    if not (rec["margin"] > MARGIN and rec["drop_margin"] > MARGIN):
        rec = oracle.incremental_block_omp(M, Y[1].astype(np.float64), c.G, 1, c.k, prev[1], 2, True, prefer=sup[1], slack=SLACK)
    assert list(sup[1]) == list(rec["support"])
    assert np.isfinite(resid[1]) and len(set(sup[1].tolist())) == c.k
    y = dev_f32(Y)
    for kwargs, args in (({}, (c.k + 1,)), ({"gamma": -1.0}, (2,))):
        with pytest.raises(binding.CsError) as e:
            cs.cs_recover_support_inc(op, dct, c.k, y, dev_i32(prev), *args, **kwargs)
        assert e.value.status == binding.CS_EINVAL
    big = binding.make_dict(None, 32, 4, 4)                      # rb > 1 is not supported by this solver
    with pytest.raises(binding.CsError) as e:
        cs.cs_recover_support_inc(binding.make_op(wl.GAUSS, 1, 0, 48, 128), big, 3, dev_f32(np.zeros((1, 48))),
                                  dev_i32(np.array([[0, 1, 2]])), 1)
    assert e.value.status == binding.CS_EINVAL


# ---- the same exchange with the inverse of the support's Gram matrix carried from token to token

def _drifting_sequence(seed, B, tokens, true_swaps):
    """Planted usage whose support drifts by `true_swaps` units per token: sketches [tokens][B][m]."""
    c = wl.CFG2
    rng = wl.rng_for(seed)
    pi, psi = wl.make_profiles(rng, c.G, c.b)
    _, S = wl.plant_usage(rng, pi, c.k, B, c.amp, c.bg)
    op = binding.make_op(c.ens, seed, 6, c.m, c.n)
    psi_dev = dev_f32(psi)
    dct = binding.make_dict(psi_dev, c.G, c.b, 1)
    M = oracle.effective_matrix(c.ens, seed, 6, c.m, c.n, c.G, c.b, 1, psi)
    first = np.stack([rng.permutation(S[t]) for t in range(B)]).astype(np.int32)
    Ys = []
    for _ in range(tokens):
        S = wl.drift_supports(rng, S, c.G, true_swaps)
        z = wl.plant_usage_on(rng, pi, S, c.amp, c.bg)
        Ys.append(oracle.sketch(c.ens, seed, 6, c.m, z).astype(np.float32))
    return c, op, dct, psi_dev, M, first, Ys


@pytest.mark.parametrize("swaps,true_swaps", [(0, 0), (2, 2), (5, 3)])
def test_carried_state_over_a_drifting_sequence(cs, swaps, true_swaps):
    """Every token starts from the support the previous call returned and from the state it left; every
    call is compared with the oracle's exchange from that same previous support."""
    B, tokens = 3, 5
    c, op, dct, psi_dev, M, prev, Ys = _drifting_sequence(4600 + swaps, B, tokens, true_swaps)
    cs.cs_plan(op, dct, psi_dev)
    state = cs.cs_inc_state(B, c.k, "cuda:0")
    exact = 0
    for t in range(tokens):
        exact += _check(cs, op, dct, M, Ys[t], c.G, c.k, prev, swaps, True, state=state)
        plain = host(cs.cs_recover_support_inc(op, dct, c.k, dev_f32(Ys[t]), dev_i32(prev), swaps)[0])
        prev = _check.last_support.copy()
        if exact == (t + 1) * B:                 # clear decisions: the two kernels agree unit for unit
            assert np.array_equal(plain, prev)
    assert exact >= B * tokens - 2
    hdr = host(state)[:, :2]
    assert np.all(hdr[:, 0] == (0x43530000 | c.k)) and np.all(hdr[:, 1] == tokens)


def test_carried_state_is_rebuilt_when_it_does_not_fit_and_when_it_is_old(cs):
    B = 2
    c, op, dct, psi_dev, M, prev, Ys = _drifting_sequence(4700, B, 70, 1)
    cs.cs_plan(op, dct, psi_dev)
    state = cs.cs_inc_state(B, c.k, "cuda:0")
    ages = []
    for t in range(70):
        sup = cs.cs_recover_support_inc_carry(op, dct, c.k, dev_f32(Ys[t]), dev_i32(prev), 1, state)[0]
        plain = cs.cs_recover_support_inc(op, dct, c.k, dev_f32(Ys[t]), dev_i32(prev), 1)[0]
        if t % 10 == 9 or t >= 63:               # the oracle on a sample of the tokens, around the rebuild
            _check(cs, op, dct, M, Ys[t], c.G, c.k, prev, 1, True, state=state.clone())
        assert np.array_equal(host(sup), host(plain)), t
        prev = host(sup)
        ages.append(int(host(state)[0, 1]))
    assert ages[:64] == list(range(1, 65)) and ages[64] == 1      # built again after 64 tokens
    # a previous support the state was not left for: the state is ignored and replaced
    other = np.stack([np.sort(wl.rng_for(1).permutation(c.G)[:c.k]) for _ in range(B)]).astype(np.int32)
    got = cs.cs_recover_support_inc_carry(op, dct, c.k, dev_f32(Ys[0]), dev_i32(other), 3, state)
    want = cs.cs_recover_support_inc(op, dct, c.k, dev_f32(Ys[0]), dev_i32(other), 3)
    assert np.array_equal(host(got[0]), host(want[0]))
    assert np.allclose(host(got[2]), host(want[2]), rtol=0, atol=RES_TOL * np.linalg.norm(Ys[0], axis=1).max())
    assert np.all(host(state)[:, 1] == 1)


def test_carried_state_full_budget_heads_and_failed_rows(cs):
    # swaps == k: nothing of the state is used, the result is recovery from nothing
    B = 3
    c, op, dct, psi_dev, M, prev, Ys = _drifting_sequence(4800, B, 2, 2)
    cs.cs_plan(op, dct, psi_dev)
    state = cs.cs_inc_state(B, c.k, "cuda:0")
    cs.cs_recover_support_inc_carry(op, dct, c.k, dev_f32(Ys[0]), dev_i32(prev), 2, state)
    ref = cs.cs_recover_support(op, dct, c.k, dev_f32(Ys[1]))
    got = cs.cs_recover_support_inc_carry(op, dct, c.k, dev_f32(Ys[1]), dev_i32(prev), c.k, state)
    assert np.array_equal(host(got[0]), host(ref[0]))
    # a failed row clears its state and leaves the other rows alone
    bad = host(got[0]).copy()
    bad[1, 3] = bad[1, 4]
    sup, coef, resid, margin = cs.cs_recover_support_inc_carry(op, dct, c.k, dev_f32(Ys[1]), dev_i32(bad), 1, state)
    assert np.all(host(sup)[1] == -1) and np.isnan(host(resid)[1]) and host(state)[1, 0] == 0
    assert host(state)[0, 0] == (0x43530000 | c.k) and np.isfinite(host(resid)[0])
    with pytest.raises(binding.CsError) as e:
        cs.cs_recover_support_inc_carry(op, dct, c.k, dev_f32(Ys[1]), dev_i32(prev), 1, None)
    assert e.value.status == binding.CS_EINVAL
    # identity dictionary (head selection), raw scores
    hs = wl.CFG3_HEADS
    rng = wl.rng_for(4810)
    _, S = wl.plant_head_usage(rng, hs, 4)
    hop = binding.make_op(hs.ens, 4810, 3, hs.m, hs.H)
    hd = binding.make_dict(None, hs.H, 1, 1)
    Mh = oracle.effective_matrix(hs.ens, 4810, 3, hs.m, hs.H, hs.H, 1, 1, None)
    hstate = cs.cs_inc_state(4, hs.kh, "cuda:0")
    prevh = S.astype(np.int32)
    for t in range(3):
        S = wl.drift_supports(rng, S, hs.H, 2)
        u = hs.bg * rng.standard_normal((4, hs.H))
        for i in range(4):
            u[i, S[i]] += rng.standard_normal(hs.kh)
        Y = oracle.sketch(hs.ens, 4810, 3, hs.m, u.astype(np.float32)).astype(np.float32)
        _check(cs, hop, hd, Mh, Y, hs.H, hs.kh, prevh, 2, False, state=hstate)
        prevh = _check.last_support.copy()


@pytest.mark.parametrize("G,k,m,swaps", [(128, 64, 200, 5), (128, 64, 200, 64), (9, 1, 8, 1), (9, 3, 8, 0), (70, 33, 96, 33), (512, 20, 120, 4)])
def test_carried_state_edge_shapes(cs, G, k, m, swaps):
    """The largest list the solver takes (k = 64: the padded copy of the inverse is full), a list of one,
    an odd size, the largest dictionary; identity dictionary, raw scores; three tokens in a row."""
    B = 3
    seed = 4900 + G + k
    rng = wl.rng_for(seed)
    op = binding.make_op(wl.GAUSS, seed, 2, m, G)
    dct = binding.make_dict(None, G, 1, 1)
    M = oracle.effective_matrix(wl.GAUSS, seed, 2, m, G, G, 1, 1, None)
    S = np.stack([np.sort(rng.permutation(G)[:k]) for _ in range(B)])
    prev = S.astype(np.int32)
    state = cs.cs_inc_state(B, k, "cuda:0")
    assert state.shape[1] == (2 + k + k * k + 3) // 4 * 4
    for t in range(3):
        S = wl.drift_supports(rng, S, G, min(swaps, 2, G - k))
        u = 0.01 * rng.standard_normal((B, G))
        for i in range(B):
            u[i, S[i]] += rng.standard_normal(k) + np.sign(rng.standard_normal(k))
        Y = oracle.sketch(wl.GAUSS, seed, 2, m, u.astype(np.float32)).astype(np.float32)
        _check(cs, op, dct, M, Y, G, k, prev, swaps, False, state=state)
        prev = _check.last_support.copy()
