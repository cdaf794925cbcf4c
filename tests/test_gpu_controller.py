"""GPU parity: entropy of the predictive distribution (the sensor of the measurement-budget
controller, Sec. 8.1) against the CPU oracle, and the budget it leads to."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_14156_amd import binding, workloads as wl
from gpu_util import dev_f32, host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,V,scale", [(5, 32000, 3.0), (3, 1000, 1.0), (2, 1, 1.0), (4, 1025, 30.0), (16, 128256, 2.0), (1, 7, 0.0)])
def test_entropy_matches_oracle(cs, B, V, scale):
    rng = wl.rng_for(B * 131 + V)
    L = (rng.standard_normal((B, V)) * scale).astype(np.float32)
    got = host(cs.cs_softmax_entropy(dev_f32(L)))
    want = oracle.softmax_entropy(L)
    assert got.shape == (B,)
    assert np.all(np.abs(got - want) <= 1e-5 * np.maximum(np.abs(want), 1.0))


def test_entropy_extreme_rows_and_budget(cs):
    V = 4096
    L = np.zeros((4, V), dtype=np.float32)
    L[1, 5] = 200.0                       # one certain token: every other term underflows
    L[2] = -1e30                          # huge negative logits everywhere but two places
    L[2, 0], L[2, 1] = np.log(0.3), np.log(0.7)
    L[3] = 1e30                           # all equal and huge: still uniform
    got = host(cs.cs_softmax_entropy(dev_f32(L)))
    want = oracle.softmax_entropy(L)
    assert np.allclose(got, want, atol=2e-5)
    assert abs(got[0] - np.log(V)) < 1e-4 and abs(got[1]) < 1e-6
    # controller: a confident step keeps the base budget, an uncertain one gets more rows
    m = [cs.cs_uds_budget(128, 0.25, float(h), 64, 512) for h in got]
    assert m == [oracle.uds_budget(128, 0.25, float(np.float32(h)), 64, 512) for h in got]
    assert m[1] == 128 and m[0] == int(np.floor(128 * (1 + 0.25 * float(np.float32(got[0])))))
    with pytest.raises(binding.CsError) as e:
        cs.cs_softmax_entropy(torch.empty((2, 0), dtype=torch.float32, device="cuda:0"))
    assert e.value.status == binding.CS_EINVAL
    assert cs.cs_softmax_entropy(torch.empty((0, 16), dtype=torch.float32, device="cuda:0")).shape == (0,)
