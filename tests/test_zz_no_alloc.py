"""The entry point that allocates nothing (cs_block_ffn_static) against cs_block_ffn, through the C ABI:
two calls in a row on the same GPU, the second with a smaller input, so that whatever the first call left
in the shared static workspace is there when the second runs."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_14156_amd import binding, workloads as wl
from gpu_util import dev_bf16, dev_i32, host, rel_err, max_abs_over_rms

pytestmark = pytest.mark.gpu


def _inputs(seed, G, b, d, k, T):
    rng = wl.rng_for(seed)
    Wg, Wu, Wd = wl.make_ffn_weights(rng, G, b, d, 0.05, "bf16")
    x = wl.make_tokens(rng, T, d, "bf16")
    sup = wl.random_supports(rng, G, k, T)
    return (Wg, Wu, Wd, x, sup), [dev_bf16(Wg), dev_bf16(Wu), dev_bf16(Wd), dev_bf16(x), dev_i32(sup)]


def test_static_workspace_entry_matches_the_allocating_one(cs):
    big_h, big = _inputs(9100, 48, 64, 1024, 12, 16)
    small_h, small = _inputs(9101, 10, 64, 256, 3, 5)
    free_before = torch.cuda.mem_get_info()[0]
    outs = []
    for dev in (big, small):                                    # two calls in a row, the second smaller
        out = torch.full_like(dev[3], float("nan"))
        cs.cs_block_ffn_static(*dev, False, out)
        outs.append(out)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] >= free_before - (8 << 20)          # nothing beyond the two outputs
    for (Wg, Wu, Wd, x, sup), dev, out in ((big_h, big, outs[0]), (small_h, small, outs[1])):
        ref = cs.cs_block_ffn(*dev, False)
        assert torch.equal(out, ref)                            # same kernels, same bits
        want = oracle.block_ffn(Wg, Wu, Wd, x, sup)
        got = host(out)
        for t in range(x.shape[0]):
            assert rel_err(got[t], want[t]) <= 2e-2 and max_abs_over_rms(got[t], want[t]) <= 2e-2, t


def test_static_workspace_limit_is_reported(cs):
    # 600 rows take the many-row path, whose workspace is far beyond the static array
    (Wg, Wu, Wd, x, sup), dev = _inputs(9102, 160, 64, 512, 150, 600)
    out = torch.empty_like(dev[3])
    with pytest.raises(binding.CsError) as e:
        cs.cs_block_ffn_static(*dev, False, out)
    assert e.value.status == binding.CS_ENOMEM and "static workspace" in str(e.value)
    # the allocating entry point serves the same call
    cs.cs_block_ffn(*dev, False)
