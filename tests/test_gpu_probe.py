"""The diagnostic streaming read: its checksum is the xor of the buffer's words (so every word was read
exactly once), for sizes below one pass, ragged sizes and a size that needs the grid-stride loop."""
import numpy as np
import pytest
import torch

from paper_2604_14156_amd import binding

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("words", [4, 4 * 37, 4 * 1024 * 8 * 3 + 4 * 11, 4 * 1024 * 8 * 1024 + 4 * 1000, 6])
def test_stream_read_checksum(cs, words):
    gen = torch.Generator(device="cuda:0").manual_seed(words)
    src = torch.randint(-2**31, 2**31 - 1, (words,), generator=gen, device="cuda:0", dtype=torch.int32)
    chk = torch.zeros((1,), dtype=torch.int32, device="cuda:0")
    cs.cs_stream_read(src, chk)
    torch.cuda.synchronize()
    host = src.cpu().numpy().view(np.uint32)
    want = np.bitwise_xor.reduce(host[: (words // 4) * 4]) if words >= 4 else np.uint32(0)
    assert np.uint32(chk.cpu().numpy().view(np.uint32)[0]) == np.uint32(want)


def test_stream_read_errors(cs):
    src = torch.zeros((64,), dtype=torch.int32, device="cuda:0")
    chk = torch.zeros((1,), dtype=torch.int32, device="cuda:0")
    with pytest.raises(binding.CsError) as e:
        cs.cs_stream_read(src[1:], chk)
    assert e.value.status == binding.CS_EALIGN
    cs.cs_stream_read(src[:0], chk)                       # nothing to read
