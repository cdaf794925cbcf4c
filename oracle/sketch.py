"""Sketch y = Phi z (the measurement equation of Sec. 3 / Sec. 8), fp64."""
import numpy as np
from .operator import phi_matrix


def sketch(ens, seed, stream_id, m, z, col_chunk=4096):
    """z: [B, n] (or [n]) -> y: [B, m].  Columns are visited in ascending order;
    the operator is materialised one column slab at a time (oracle only)."""
    z = np.asarray(z, dtype=np.float64)
    single = z.ndim == 1
    z2 = z[None, :] if single else z
    B, n = z2.shape
    y = np.zeros((B, m), dtype=np.float64)
    for c0 in range(0, n, col_chunk):
        nc = min(col_chunk, n - c0)
        phi = phi_matrix(ens, seed, stream_id, m, n, c0, nc)     # [m, nc]
        y += z2[:, c0:c0 + nc] @ phi.T
    return y[0] if single else y
