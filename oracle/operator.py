"""Random measurement operator Phi (the paper's A_t, Sec. 3 and Sec. 8).

The paper asks only for a random or pseudo-random m x n matrix from a
subgaussian ensemble.  Here every entry is a pure function of
(seed, stream_id, row, col), so the matrix never has to be stored and its rows
are nested: changing the measurement budget m (Sec. 8.1) adds or removes rows
and rescales, nothing else.

Entry convention (this project's own; both ensembles use Philox4x32-10):
  key     = (seed mod 2**32, seed >> 32)
  counter = (col // cols_per_call, row, stream_id, ensemble)
  Rademacher (ensemble 1): one call yields 128 sign bits; column c uses bit
      (c mod 32) of output word ((c mod 128) // 32); bit 0 -> +1, bit 1 -> -1.
  Gaussian (ensemble 0): one call yields 4 normals by Box-Muller; with
      p = (c mod 4) // 2, u1 = (w[2p]+1) / 2**32, u2 = (w[2p+1]+1) / 2**32,
      rad = sqrt(-2 ln u1): even columns take rad*cos(2 pi u2), odd columns
      rad*sin(2 pi u2).
  Phi[row, col] = entry / sqrt(m).
"""
import numpy as np
from .philox import philox4x32_10

GAUSS = 0
RADEMACHER = 1


def phi_entries(ens, seed, stream_id, rows, cols):
    """Unscaled entries e(row, col), fp64, for index arrays that broadcast."""
    rows = np.asarray(rows, dtype=np.uint64)
    cols = np.asarray(cols, dtype=np.uint64)
    rows, cols = np.broadcast_arrays(rows, cols)
    k0 = np.uint64(seed & 0xFFFFFFFF)
    k1 = np.uint64((seed >> 32) & 0xFFFFFFFF)
    if ens == RADEMACHER:
        w = philox4x32_10(cols // np.uint64(128), rows, stream_id, RADEMACHER, k0, k1)
        t = cols % np.uint64(128)
        word = np.choose((t // np.uint64(32)).astype(np.int64), w)
        bit = (word >> (t % np.uint64(32)).astype(np.uint32)) & np.uint32(1)
        return 1.0 - 2.0 * bit.astype(np.float64)
    if ens == GAUSS:
        w = philox4x32_10(cols // np.uint64(4), rows, stream_id, GAUSS, k0, k1)
        p = ((cols % np.uint64(4)) // np.uint64(2)).astype(np.int64)
        wa = np.choose(p, (w[0], w[2])).astype(np.float64)
        wb = np.choose(p, (w[1], w[3])).astype(np.float64)
        u1 = (wa + 1.0) / 4294967296.0
        u2 = (wb + 1.0) / 4294967296.0
        rad = np.sqrt(-2.0 * np.log(u1))
        ang = 2.0 * np.pi * u2
        odd = (cols % np.uint64(2)).astype(bool)
        return np.where(odd, rad * np.sin(ang), rad * np.cos(ang))
    raise ValueError("unknown ensemble")


def phi_matrix(ens, seed, stream_id, m, n, col0=0, ncols=None):
    """The scaled operator Phi (or a column slice of it) as a dense fp64 array."""
    ncols = n - col0 if ncols is None else ncols
    rows = np.arange(m, dtype=np.uint64)[:, None]
    cols = np.arange(col0, col0 + ncols, dtype=np.uint64)[None, :]
    return phi_entries(ens, seed, stream_id, rows, cols) / np.sqrt(float(m))
