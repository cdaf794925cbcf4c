import os
import sys
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def cs():
    """The ctypes binding over the HIP library, with a context on cuda:0.  Result buffers that the
    binding allocates sit between guard bands, verified after every call (gpu_util.guarded_context)."""
    import torch
    import gpu_util
    if not torch.cuda.is_available():
        pytest.fail("GPU test collected on a machine without a GPU")
    ctx = gpu_util.guarded_context(0)
    yield ctx
    # every buffer the binding allocated for a result was checked (a selection of tests that lets the caller
    # allocate all outputs allocates none)
    assert ctx.guards_checked >= ctx.guards_allocated - len(ctx._pending)
    assert ctx.guards_allocated == 0 or ctx.guards_checked > 0
    ctx.close()
