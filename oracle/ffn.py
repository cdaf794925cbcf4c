"""Block-sparse SwiGLU feed-forward layer (oracle, fp64).

Sec. 3 defines reduced execution as the dense operator with every unit outside
the support masked off.  For a gated FFN whose d_ff channels are split into G
blocks of b channels, a channel c in an active block contributes
    h_c = silu(<Wg_c, x>) * <Wu_c, x>,     out += h_c * Wd_c,
with silu(t) = t / (1 + exp(-t)); channels of inactive blocks contribute 0.
"""
import numpy as np


def block_ffn(Wg, Wu, Wd, x, support):
    """Wg, Wu: [G, b, d] (channel-major rows).  Wd: [G, d, b] (the block's slice
    of the down projection, stored output-row-major).  x: [T, d].
    support: [k] shared by all rows of x, or [T, k] one per row.
    Returns out [T, d] in fp64 (no rounding of the result)."""
    Wg = np.asarray(Wg, dtype=np.float64)
    Wu = np.asarray(Wu, dtype=np.float64)
    Wd = np.asarray(Wd, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    T, d = x.shape
    support = np.asarray(support)
    out = np.zeros((T, d), dtype=np.float64)
    for t in range(T):
        units = support if support.ndim == 1 else support[t]
        for g in units:
            gate = Wg[g] @ x[t]                       # [b]
            up = Wu[g] @ x[t]
            h = gate / (1.0 + np.exp(-gate)) * up
            out[t] += Wd[g] @ h                       # [d, b] @ [b]
    return out
