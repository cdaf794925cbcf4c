"""Helpers for the GPU parity tests: host<->device transfer and error measures."""
import numpy as np
import torch

DEV = "cuda:0"


def dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def dev_bf16(a):
    # `a` already holds bf16-representable values, so this conversion is exact
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV).to(torch.bfloat16)


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def dev_w(a, dtype):
    return dev_bf16(a) if dtype == "bf16" else dev_f32(a)


def host(t):
    torch.cuda.synchronize()
    return t.detach().float().cpu().numpy().astype(np.float64) if t.is_floating_point() else t.cpu().numpy()


def rel_err(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    denom = np.linalg.norm(want)
    return np.linalg.norm(got - want) / (denom if denom > 0 else 1.0)


def max_abs_over_rms(got, want):
    """Largest element error of a row in units of the reference row's root mean square."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    rms = np.sqrt(np.mean(want ** 2))
    return float(np.max(np.abs(got - want)) / (rms if rms > 0 else 1.0))


GUARD_BYTES = 256
GUARD_FILL = 0xA5


def guarded_context(device=0):
    """A binding context whose own output allocations carry guard bands.

    Every buffer the binding allocates for a call's results is a window into a larger byte buffer filled
    with a marker; after each library call the stream is synchronised and the 256 bytes before and after
    every such window must still hold the marker, else the call wrote outside an output buffer."""
    from paper_2604_14156_amd import binding

    class GuardedContext(binding.Context):
        def __init__(self, device):
            super().__init__(device=device)
            self._pending = []
            self.guards_allocated = 0
            self.guards_checked = 0

        def _alloc(self, shape, dtype, device):
            n = 1
            for s in shape:
                n *= int(s)
            nbytes = n * torch.empty((), dtype=dtype).element_size()
            raw = torch.full((2 * GUARD_BYTES + nbytes,), GUARD_FILL, dtype=torch.uint8, device=device)
            self._pending.append((raw, nbytes))
            self.guards_allocated += 1
            return raw[GUARD_BYTES:GUARD_BYTES + nbytes].view(dtype).view(tuple(shape))

        def _check(self, st):
            pending, self._pending = self._pending, []
            torch.cuda.synchronize()
            for raw, nbytes in pending:
                front = raw[:GUARD_BYTES]
                back = raw[GUARD_BYTES + nbytes:]
                ok = bool((front == GUARD_FILL).all()) and bool((back == GUARD_FILL).all())
                assert ok, "a library call wrote outside an output buffer of %d bytes" % nbytes
                self.guards_checked += 1
            super()._check(st)

    return GuardedContext(device)


def assert_greedy_support(M, y, G, rb, k, normalised, got, rec, margin=1e-3, slack=1e-3):
    """`got` against the oracle's block-OMP result `rec` on (M, y): identical when the oracle's smallest
    selection margin is above `margin`; otherwise several supports are correct and `got` must be one of
    them, i.e. the oracle reproduces it when it prefers its units within `slack`.  Returns True when the
    comparison was the exact one."""
    import oracle
    got = [int(g) for g in got]
    if rec["margin"] > margin:
        assert got == list(rec["support"]), (rec["margin"], sorted(set(got) ^ set(rec["support"].tolist())))
        return True
    if got == list(rec["support"]):
        return False                      # a near tie resolved as the oracle's plain rule resolves it
    rep = oracle.block_omp(M, y, G, rb, k, normalised, prefer=got, slack=slack)
    assert got == list(rep["support"]), (rec["margin"], sorted(set(got) ^ set(rec["support"].tolist())))
    return False
