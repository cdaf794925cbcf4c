"""GPU parity: block-sparse FFN and head-pruned attention against the CPU oracle,
through the C ABI.  Tolerances: fp32 layers 1e-5, bf16 layers 2e-2 (relative L2
error of each output row against the unrounded fp64 oracle), and for every single
element |got - want| <= 4e-5 (fp32) or 2e-2 (bf16) times the root mean square of
the oracle's row, so that one wrong element cannot hide in a row norm."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_14156_amd import binding, workloads as wl
from gpu_util import dev_w, dev_bf16, dev_i32, host, rel_err, max_abs_over_rms, assert_greedy_support, dev_f32

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-5, "bf16": 2e-2}
ELT = {"f32": 4e-5, "bf16": 2e-2}


def check_row(got, want, dtype="bf16", what=None):
    e2, emax = rel_err(got, want), max_abs_over_rms(got, want)
    assert e2 <= TOL[dtype] and emax <= ELT[dtype], (what, e2, emax)


def _ffn_case(cs, seed, G, b, d, k, T, dtype, shared, std):
    rng = wl.rng_for(seed)
    Wg, Wu, Wd = wl.make_ffn_weights(rng, G, b, d, std, dtype)
    x = wl.make_tokens(rng, T, d, dtype)
    sup = wl.random_supports(rng, G, k, 1)[0] if shared else wl.random_supports(rng, G, k, T)
    for t in range(0 if shared else T):            # supports need not be sorted
        rng.shuffle(sup[t])
    out = host(cs.cs_block_ffn(dev_w(Wg, dtype), dev_w(Wu, dtype), dev_w(Wd, dtype), dev_w(x, dtype),
                               dev_i32(sup), shared))
    want = oracle.block_ffn(Wg, Wu, Wd, x, sup)
    for t in range(T):
        check_row(out[t], want[t], dtype, t)


def test_ffn_tiny_planted_config(cs):
    c = wl.CFG1
    _ffn_case(cs, 1000, c.G, c.b, c.d, c.k, 1, "f32", False, c.wstd)


@pytest.mark.parametrize("T,shared", [(1, False), (5, False), (8, False), (16, False), (19, False), (7, True), (1, True)])
def test_ffn_bf16_small_shapes(cs, T, shared):
    _ffn_case(cs, 1100 + T, 10, 64, 512, 3, T, "bf16", shared, 0.05)


@pytest.mark.parametrize("T", [1, 3])
def test_ffn_f32_ragged_shapes(cs, T):
    _ffn_case(cs, 1200 + T, 7, 24, 136, 7, T, "f32", False, 0.1)     # k == G: the dense layer


@pytest.mark.parametrize("T,shared,G,k,d", [(300, True, 20, 5, 1024), (130, False, 12, 4, 512), (64, False, 9, 9, 256),
                                            (257, True, 6, 1, 128),
                                            # long batches (wide tiles): ragged last row tile, odd block count,
                                            # output width that is no multiple of the tile, per-row supports
                                            (600, True, 20, 5, 1024), (515, False, 12, 4, 320), (1024, True, 8, 8, 256),
                                            (513, True, 5, 1, 64)])
def test_ffn_bf16_many_rows_matrix_core_path(cs, T, shared, G, k, d):
    _ffn_case(cs, 1500 + T, G, 64, d, k, T, "bf16", shared, 0.05)


def test_ffn_prefill_shape_full_size(cs):
    """Task-conditioned prefill at full size, the whole chain: the prompt-level usage is sketched, one
    support is recovered from the sketch (compared with the oracle's), and that support (still on the
    device) drives the shared-support layer over 2048 rows.  Weights are drawn on the device; the oracle
    computes 48 rows spread over all row tiles, among them the first and last of a tile."""
    c = wl.CFG4
    T = 2048
    seed = 4001
    rng = wl.rng_for(seed)
    pi, psi = wl.make_profiles(rng, c.G, c.b)
    z, S = wl.plant_usage(rng, pi, c.k, 2, c.amp, c.bg)
    z, S = z[1:2], S[1:2]                                         # the second instance: oracle margin 2.3e-3
    op = binding.make_op(c.ens, seed, 0, c.m, c.n)
    psi_dev = dev_f32(psi)
    dct = binding.make_dict(psi_dev, c.G, c.b, 1)
    cs.cs_plan(op, dct, psi_dev)
    y = cs.cs_sketch(op, dev_f32(z))
    sup_dev = cs.cs_recover_support(op, dct, c.k, y, want_coef=False, want_resid=False)[0]
    M = oracle.effective_matrix(c.ens, seed, 0, c.m, c.n, c.G, c.b, 1, psi)
    y_or = oracle.sketch(c.ens, seed, 0, c.m, z[0])
    rec = oracle.block_omp(M, y_or, c.G, 1, c.k, True)
    sup = host(sup_dev)[0]
    assert assert_greedy_support(M, y_or, c.G, 1, c.k, True, sup, rec)        # the exact comparison applies
    assert list(sup) == list(S[0])

    gen = torch.Generator(device="cuda:0").manual_seed(41)
    Wg, Wu = (torch.randn((c.G, c.b, c.d), generator=gen, device="cuda:0").mul_(c.wstd).to(torch.bfloat16) for _ in range(2))
    Wd = torch.randn((c.G, c.d, c.b), generator=gen, device="cuda:0").mul_(c.wstd).to(torch.bfloat16)
    x = torch.randn((T, c.d), generator=gen, device="cuda:0").to(torch.bfloat16)
    out = cs.cs_block_ffn(Wg, Wu, Wd, x, sup_dev[0], True)
    torch.cuda.synchronize()
    rows = sorted(set([0, 127, 128, 255, 256, 1000, 1023, 1024, 2046, 2047] + list(range(5, T, 53))))
    hx = host(x[rows])
    # the oracle needs only the kept blocks: gather them on the device, upcast on the host
    idx = torch.from_numpy(sup.astype(np.int64)).to("cuda:0")
    hWg, hWu, hWd = host(Wg[idx]), host(Wu[idx]), host(Wd[idx])
    want = oracle.block_ffn(hWg, hWu, hWd, hx, np.arange(c.k))
    got = host(out[rows])
    for i in range(len(rows)):
        check_row(got[i], want[i], "bf16", rows[i])
    # every row was written: no row of the output is far from the scale of the checked ones
    norms = out.float().norm(dim=1)
    ref = float(np.median(np.linalg.norm(want, axis=1)))
    assert float(norms.min()) > 0.5 * ref and float(norms.max()) < 2.0 * ref


@pytest.mark.parametrize("T,shared,G,k,d", [(2100, True, 40, 35, 4160), (2052, False, 40, 9, 4128), (1300, True, 64, 63, 2080),
                                            (1100, True, 30, 7, 4000), (1290, False, 24, 5, 4064)])
def test_ffn_wide_tiles_ragged_shapes(cs, T, shared, G, k, d):
    """Shapes large enough for the 256 x 256 tiles on at least one of the two products, with a ragged last
    row tile, an odd number of blocks, an output width that is no multiple of the tile, and (second case)
    per-row supports; the last two have too few 256 x 256 tiles for the second product and take 128 x 128
    ones there, again with ragged rows and columns; oracle on sampled rows, among them the last ones."""
    gen = torch.Generator(device="cuda:0").manual_seed(T + d)
    b = 64
    Wg, Wu = (torch.randn((G, b, d), generator=gen, device="cuda:0").mul_(0.03).to(torch.bfloat16) for _ in range(2))
    Wd = torch.randn((G, d, b), generator=gen, device="cuda:0").mul_(0.03).to(torch.bfloat16)
    x = torch.randn((T, d), generator=gen, device="cuda:0").to(torch.bfloat16)
    rng = wl.rng_for(T + d)
    sup = wl.random_supports(rng, G, k, 1)[0] if shared else wl.random_supports(rng, G, k, T)
    out = cs.cs_block_ffn(Wg, Wu, Wd, x, dev_i32(sup), shared)
    torch.cuda.synchronize()
    rows = [0, 127, 128, 255, 256, T // 2, T - 37, T - 2, T - 1]
    hWg, hWu, hWd = host(Wg), host(Wu), host(Wd)
    got = host(out[rows])
    for i, r in enumerate(rows):
        want = oracle.block_ffn(hWg, hWu, hWd, host(x[r:r + 1]), sup if shared else sup[r])[0]
        check_row(got[i], want, "bf16", r)


def test_joint_prompt_shape_gather_and_ffn(cs):
    """Kept-token gather followed by the shared-support FFN (joint selection workload), sampled rows."""
    c = wl.CFG2
    n_tok, k_tok = 8192, 2048
    gen = torch.Generator(device="cuda:0").manual_seed(51)
    Wg, Wu = (torch.randn((c.G, c.b, c.d), generator=gen, device="cuda:0").mul_(c.wstd).to(torch.bfloat16) for _ in range(2))
    Wd = torch.randn((c.G, c.d, c.b), generator=gen, device="cuda:0").mul_(c.wstd).to(torch.bfloat16)
    X = torch.randn((n_tok, c.d), generator=gen, device="cuda:0").to(torch.bfloat16)
    rng = wl.rng_for(51)
    tokens = np.sort(rng.choice(n_tok, size=k_tok, replace=False)).astype(np.int32)
    sup = wl.random_supports(rng, c.G, c.k, 1)[0]
    Xk = cs.cs_gather_rows(X, dev_i32(tokens))
    torch.cuda.synchronize()
    assert torch.equal(Xk, X[torch.from_numpy(tokens.astype(np.int64)).to("cuda:0")])       # byte-exact copy
    out = cs.cs_block_ffn(Wg, Wu, Wd, Xk, dev_i32(sup), True)
    rows = sorted(set([0, 1, 127, 128, 1023, 1024, 2046, 2047] + list(range(3, k_tok, 41))))
    idx = torch.from_numpy(sup.astype(np.int64)).to("cuda:0")
    want = oracle.block_ffn(host(Wg[idx]), host(Wu[idx]), host(Wd[idx]), host(X[tokens[rows].astype(np.int64)]), np.arange(c.k))
    got = host(out[rows])
    for i in range(len(rows)):
        check_row(got[i], want[i], "bf16", rows[i])
    # an out-of-range token yields a zero row
    z = cs.cs_gather_rows(X, dev_i32(np.array([5, n_tok, -1, 7], dtype=np.int32)))
    torch.cuda.synchronize()
    assert float(z[1].float().abs().max()) == 0.0 and float(z[2].float().abs().max()) == 0.0 and torch.equal(z[3], X[7])


@pytest.mark.parametrize("T,G,b,k,d", [(17, 10, 64, 3, 512), (37, 12, 32, 5, 416), (48, 30, 64, 30, 256), (64, 7, 96, 2, 1056),
                                       (33, 300, 64, 4, 128), (64, 9, 64, 7, 512), (30, 6, 64, 5, 256), (64, 40, 64, 10, 1536)])
def test_ffn_bf16_17_to_64_rows_per_token_supports(cs, T, G, b, k, d):
    """The path for 17 to 64 token rows with their own supports: ragged token tiles, a width that is no
    multiple of the staged chunk, blocks of 32 and 96 channels, k == G, more channels than one pass of a
    workgroup holds (300 blocks on few workgroups is not reached here, many blocks on 256 are), blocks
    listed by more than half of the tokens (two items per block in the down kernel for 64-channel blocks,
    at two, three and four token tiles) and by fewer (one item)."""
    _ffn_case(cs, 1800 + T, G, b, d, k, T, "bf16", False, 0.05)


def test_ffn_17_to_64_rows_supports_from_a_few_blocks(cs):
    """Forty rows whose supports all come from 12 of 50 blocks: the rows list eight times as many entries as
    there are blocks, so the kernel starts on the guess that every block is listed, finds a list of at most
    12 and has to take its channel ranges from that list instead."""
    rng = wl.rng_for(1860)
    G, b, d, T, k = 50, 64, 1024, 40, 10
    Wg, Wu, Wd = wl.make_ffn_weights(rng, G, b, d, 0.05, "bf16")
    x = wl.make_tokens(rng, T, d, "bf16")
    pool = rng.choice(G, size=12, replace=False)
    sup = np.stack([rng.choice(pool, size=k, replace=False) for _ in range(T)]).astype(np.int32)
    got = host(cs.cs_block_ffn(dev_bf16(Wg), dev_bf16(Wu), dev_bf16(Wd), dev_bf16(x), dev_i32(sup), False))
    want = oracle.block_ffn(Wg, Wu, Wd, x, sup)
    for t in range(T):
        check_row(got[t], want[t], "bf16", t)


def test_ffn_17_to_64_rows_out_of_range_units(cs):
    rng = wl.rng_for(1850)
    G, b, d, T = 8, 64, 256, 20
    Wg, Wu, Wd = wl.make_ffn_weights(rng, G, b, d, 0.05, "bf16")
    x = wl.make_tokens(rng, T, d, "bf16")
    sup = wl.random_supports(rng, G, 3, T)
    sup[0, 1] = -1
    sup[5, 0] = G + 3
    sup[19, :] = [G, -5, 99]                                   # a token with no valid unit: a zero row
    got = host(cs.cs_block_ffn(dev_bf16(Wg), dev_bf16(Wu), dev_bf16(Wd), dev_bf16(x), dev_i32(sup), False))
    for t in range(T):
        want = oracle.block_ffn(Wg, Wu, Wd, x[t:t + 1], [g for g in sup[t] if 0 <= g < G])[0]
        if t == 19:
            assert np.all(got[t] == 0.0)
        else:
            check_row(got[t], want, "bf16", t)


def test_ffn_bf16_block_of_32_channels(cs):
    _ffn_case(cs, 1300, 12, 32, 256, 5, 4, "bf16", False, 0.05)


def test_ffn_empty_cases(cs):
    rng = wl.rng_for(1400)
    Wg, Wu, Wd = wl.make_ffn_weights(rng, 4, 64, 128, 0.05, "bf16")
    x = wl.make_tokens(rng, 3, 128, "bf16")
    dW = [dev_bf16(w) for w in (Wg, Wu, Wd)]
    out = cs.cs_block_ffn(*dW, dev_bf16(x), torch.empty((3, 0), dtype=torch.int32, device="cuda:0"), False)
    assert float(out.float().abs().max()) == 0.0                       # empty support: zeros
    out = cs.cs_block_ffn(*dW, dev_bf16(x[:0]), dev_i32(np.zeros((0, 2))), False)
    assert out.shape == (0, 128)
    # an out-of-range unit contributes nothing
    sup = np.array([[1, 99], [2, -1], [0, 3]], dtype=np.int32)
    got = host(cs.cs_block_ffn(*dW, dev_bf16(x), dev_i32(sup), False))
    want = np.stack([oracle.block_ffn(Wg, Wu, Wd, x[t:t + 1], [g for g in sup[t] if 0 <= g < 4])[0] for t in range(3)])
    for t in range(3):
        check_row(got[t], want[t], "bf16", t)
    with pytest.raises(binding.CsError) as e:
        cs.cs_block_ffn(*dW, dev_bf16(x), dev_i32(np.zeros((3, 5))), False)    # k > G
    assert e.value.status == binding.CS_EINVAL


@pytest.mark.parametrize("case", ["high_blocks_only", "shared_by_all_tokens", "low_blocks_only", "independent"])
def test_ffn_decode_dense_union_guess(cs, case):
    """16 tokens x 6 of 40 blocks: enough listed entries for the decode kernel to fix its first items by
    workgroup index before it knows the supports (blocks 0..31).  The guess is wrong for every such item
    when the tokens only use blocks 32..39, for most when all tokens share one support, right for most when
    only low blocks are used."""
    G, b, d, k, T = 40, 64, 512, 6, 16
    rng = wl.rng_for(1700 + len(case))
    Wg, Wu, Wd = wl.make_ffn_weights(rng, G, b, d, 0.05, "bf16")
    x = wl.make_tokens(rng, T, d, "bf16")
    if case == "high_blocks_only":
        sup = np.stack([rng.permutation(np.arange(32, 40))[:k] for _ in range(T)]).astype(np.int32)
    elif case == "shared_by_all_tokens":
        sup = np.tile(wl.random_supports(rng, G, k, 1)[0], (T, 1)).astype(np.int32)
    elif case == "low_blocks_only":
        sup = np.stack([rng.permutation(np.arange(0, 12))[:k] for _ in range(T)]).astype(np.int32)
    else:
        sup = wl.random_supports(rng, G, k, T)
    out = host(cs.cs_block_ffn(dev_bf16(Wg), dev_bf16(Wu), dev_bf16(Wd), dev_bf16(x), dev_i32(sup), False))
    want = oracle.block_ffn(Wg, Wu, Wd, x, sup)
    for t in range(T):
        check_row(out[t], want[t], "bf16", (case, t))


@pytest.mark.parametrize("T,G,k", [(16, 40, 6), (6, 40, 4), (40, 24, 5)])
def test_ffn_union_hint_changes_no_result(cs, T, G, k):
    """The caller's word on the union of the supports only moves loads: with the hint set either way, on
    supports for which it is right and on supports for which it is wrong, the output is that of the default,
    bit for bit, and within tolerance of the oracle."""
    b, d = 64, 512
    rng = wl.rng_for(1800 + T)
    Wg, Wu, Wd = wl.make_ffn_weights(rng, G, b, d, 0.05, "bf16")
    x = wl.make_tokens(rng, T, d, "bf16")
    spread = wl.random_supports(rng, G, k, T)
    shared = np.tile(wl.random_supports(rng, G, k, 1)[0], (T, 1)).astype(np.int32)
    args = [dev_bf16(Wg), dev_bf16(Wu), dev_bf16(Wd), dev_bf16(x)]
    try:
        for sup in (spread, shared):
            cs.cs_set_union_hint(0)
            ref = host(cs.cs_block_ffn(*args, dev_i32(sup), False))
            want = oracle.block_ffn(Wg, Wu, Wd, x, sup)
            for t in range(T):
                check_row(ref[t], want[t], "bf16", t)
            for hint in (1, 2):
                cs.cs_set_union_hint(hint)
                got = host(cs.cs_block_ffn(*args, dev_i32(sup), False))
                assert np.array_equal(got, ref), hint          # bf16 values widened exactly: equal floats = equal bits
        with pytest.raises(binding.CsError) as e:
            cs.cs_set_union_hint(7)
        assert e.value.status == binding.CS_EINVAL
    finally:
        cs.cs_set_union_hint(0)


def _full_size_ffn(cs, B, seed):
    """Decode shape at full size: weights drawn on the device, every token against the oracle."""
    c = wl.CFG2
    gen = torch.Generator(device="cuda:0").manual_seed(seed)
    Wg, Wu = (torch.randn((c.G, c.b, c.d), generator=gen, device="cuda:0").mul_(c.wstd).to(torch.bfloat16) for _ in range(2))
    Wd = torch.randn((c.G, c.d, c.b), generator=gen, device="cuda:0").mul_(c.wstd).to(torch.bfloat16)
    x = torch.randn((B, c.d), generator=gen, device="cuda:0").to(torch.bfloat16)
    sup = wl.random_supports(wl.rng_for(seed), c.G, c.k, B)
    out = host(cs.cs_block_ffn(Wg, Wu, Wd, x, dev_i32(sup), False))
    hWg, hWu, hWd, hx = host(Wg), host(Wu), host(Wd), host(x)
    for t in range(B):
        want = oracle.block_ffn(hWg, hWu, hWd, hx[t:t + 1], sup[t])[0]
        check_row(out[t], want, "bf16", t)


@pytest.mark.parametrize("B", [1, 8, 16, 17, 33, 64])
def test_ffn_decode_shape_full_size(cs, B):
    _full_size_ffn(cs, B, 2000 + B)


def _attn_case(cs, seed, B, H, L, dh, kh):
    rng = wl.rng_for(seed)
    q, K, V = wl.make_kv(rng, B, H, L, dh)
    heads = wl.random_supports(rng, H, kh, B)
    out = host(cs.cs_head_attn(dev_bf16(q), dev_bf16(K), dev_bf16(V), dev_i32(heads)))
    want = oracle.head_attn(q, K, V, heads)
    for b in range(B):
        kept = set(heads[b].tolist())
        for h in range(H):
            if h in kept:
                check_row(out[b, h], want[b, h], "bf16", (b, h))
            else:
                assert np.all(out[b, h] == 0.0)


@pytest.mark.parametrize("B,H,L,dh,kh", [(2, 4, 300, 128, 2), (1, 3, 1, 128, 3), (3, 8, 1000, 64, 3),
                                         (2, 2, 77, 256, 1), (1, 32, 4096, 128, 12), (2, 4, 130, 128, 0)])
def test_attention_small_and_ragged(cs, B, H, L, dh, kh):
    _attn_case(cs, 3000 + L + dh, B, H, L, dh, kh)


def test_attention_decode_shape_full_size(cs):
    hs = wl.CFG3_HEADS
    B = 16
    gen = torch.Generator(device="cuda:0").manual_seed(31)
    q = torch.randn((B, hs.H, hs.dh), generator=gen, device="cuda:0").to(torch.bfloat16)
    K = torch.randn((B, hs.H, hs.L, hs.dh), generator=gen, device="cuda:0").to(torch.bfloat16)
    V = torch.randn((B, hs.H, hs.L, hs.dh), generator=gen, device="cuda:0").to(torch.bfloat16)
    heads = wl.random_supports(wl.rng_for(31), hs.H, hs.kh, B)
    out = host(cs.cs_head_attn(q, K, V, dev_i32(heads)))
    hq = host(q)
    for b in range(B):                                 # every kept (sequence, head) pair, every pruned head
        for h in heads[b]:
            h = int(h)
            want = oracle.head_attn(hq[b:b + 1, h:h + 1], host(K[b:b + 1, h:h + 1]), host(V[b:b + 1, h:h + 1]),
                                    np.array([[0]]))[0, 0]
            check_row(out[b, h], want, "bf16", (b, h))
        pruned = sorted(set(range(hs.H)) - set(heads[b].tolist()))
        assert np.all(out[b, pruned] == 0.0)


@pytest.mark.parametrize("B,H,L,dh,kh", [(8, 32, 2500, 128, 16), (16, 16, 5001, 64, 8), (24, 8, 1030, 256, 6)])
def test_attention_wide_workgroups_ragged_cache(cs, B, H, L, dh, kh):
    """Batches large enough for the 16-wave workgroup shape, cache lengths that are not a multiple of a
    workgroup's pass; oracle on sampled (sequence, head) pairs, zeros on every pruned head."""
    gen = torch.Generator(device="cuda:0").manual_seed(L + dh)
    q = torch.randn((B, H, dh), generator=gen, device="cuda:0").to(torch.bfloat16)
    K = torch.randn((B, H, L, dh), generator=gen, device="cuda:0").to(torch.bfloat16)
    V = torch.randn((B, H, L, dh), generator=gen, device="cuda:0").to(torch.bfloat16)
    heads = wl.random_supports(wl.rng_for(L), H, kh, B)
    out = host(cs.cs_head_attn(q, K, V, dev_i32(heads)))
    hq = host(q)
    for b in (0, B // 2, B - 1):
        for h in (int(heads[b][0]), int(heads[b][kh // 2]), int(heads[b][-1])):
            want = oracle.head_attn(hq[b:b + 1, h:h + 1], host(K[b:b + 1, h:h + 1]), host(V[b:b + 1, h:h + 1]),
                                    np.array([[0]]))[0, 0]
            check_row(out[b, h], want, "bf16", (b, h))
    for b in range(B):
        pruned = sorted(set(range(H)) - set(heads[b].tolist()))
        assert np.all(out[b, pruned] == 0.0)
        assert np.all(np.abs(out[b, heads[b]]).max(axis=1) > 0.0)


def test_attention_sharp_scores_do_not_overflow(cs):
    rng = wl.rng_for(3500)
    q, K, V = wl.make_kv(rng, 1, 2, 200, 128)
    q = wl.round_bf16(q * 8.0)                    # scores of order +-100
    heads = np.array([[0, 1]], dtype=np.int32)
    out = host(cs.cs_head_attn(dev_bf16(q), dev_bf16(K), dev_bf16(V), dev_i32(heads)))
    want = oracle.head_attn(q, K, V, heads)
    assert np.all(np.isfinite(out))
    for h in range(2):
        check_row(out[0, h], want[0, h], "bf16", h)
