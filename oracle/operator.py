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
  Subsampled randomised Hadamard (ensemble 2; Sec. 8 names it for implementation
      efficiency): Phi = (1/sqrt(m)) R H D on the first n columns, with H the
      Walsh-Hadamard matrix of order n' = 2**b, the smallest power of two >= max(n, 2)
      (H[r, c] = (-1)**popcount(r & c)), D a diagonal of Rademacher signs and R a
      choice of m distinct rows:
        d_c   = the Rademacher bit of column c drawn as above with counter
                (c // 128, 0, stream_id, 2);
        r_i   = perm(i), a bijection of [0, n') built from the four words w of the
                Philox call with counter (0, 1, stream_id, 2):
                x = (i * (w0 | 1) + w1) mod n';  x ^= x >> ceil(b/2);
                x = (x * (w2 | 1) + w3) mod n';  x ^= x >> ceil(b/2);
        entry(i, c) = d_c * H[r_i, c].
      Rows are nested in m like those of the other ensembles (m <= n').
  Phi[row, col] = entry / sqrt(m).
"""
import numpy as np
from .philox import philox4x32_10

GAUSS = 0
RADEMACHER = 1
SRHT = 2


def srht_order(n):
    """(n', b): order of the Hadamard matrix used for n columns and its number of index bits."""
    b = 1
    while (1 << b) < n:
        b += 1
    return 1 << b, b


def srht_rows(seed, stream_id, rows, n):
    """r_i = perm(i): the Hadamard row measured by measurement i (array in, array out)."""
    npad, b = srht_order(n)
    k0 = np.uint64(seed & 0xFFFFFFFF)
    k1 = np.uint64((seed >> 32) & 0xFFFFFFFF)
    w = philox4x32_10(np.uint64(0), np.uint64(1), stream_id, SRHT, k0, k1)
    w = [int(v) for v in w]
    mask = npad - 1
    sh = (b + 1) // 2
    out = []
    for i in np.asarray(rows, dtype=np.int64).reshape(-1):
        x = (int(i) * (w[0] | 1) + w[1]) & mask
        x ^= x >> sh
        x = (x * (w[2] | 1) + w[3]) & mask
        x ^= x >> sh
        out.append(x)
    return np.array(out, dtype=np.uint64).reshape(np.shape(rows))


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
    raise ValueError("unknown ensemble (the Hadamard ensemble needs the column count: use phi_matrix)")


def srht_entries(seed, stream_id, rows, cols, n):
    """Unscaled entries d_c * H[r_i, c] of the subsampled randomised Hadamard operator on n columns."""
    rows = np.asarray(rows, dtype=np.uint64)
    cols = np.asarray(cols, dtype=np.uint64)
    k0 = np.uint64(seed & 0xFFFFFFFF)
    k1 = np.uint64((seed >> 32) & 0xFFFFFFFF)
    r = srht_rows(seed, stream_id, rows, n)
    r, c = np.broadcast_arrays(r, cols)
    w = philox4x32_10(c // np.uint64(128), np.zeros_like(c), stream_id, SRHT, k0, k1)
    t = c % np.uint64(128)
    word = np.choose((t // np.uint64(32)).astype(np.int64), w)
    dbit = ((word >> (t % np.uint64(32)).astype(np.uint32)) & np.uint32(1)).astype(np.int64)
    v = (r & c).astype(np.uint64)
    par = np.zeros(v.shape, dtype=np.int64)
    for s in range(32):                                  # parity of popcount(r & c); indices are below 2**32
        par ^= ((v >> np.uint64(s)) & np.uint64(1)).astype(np.int64)
    return 1.0 - 2.0 * ((par ^ dbit) & 1).astype(np.float64)


def phi_matrix(ens, seed, stream_id, m, n, col0=0, ncols=None):
    """The scaled operator Phi (or a column slice of it) as a dense fp64 array."""
    ncols = n - col0 if ncols is None else ncols
    rows = np.arange(m, dtype=np.uint64)[:, None]
    cols = np.arange(col0, col0 + ncols, dtype=np.uint64)[None, :]
    if ens == SRHT:
        if m > srht_order(n)[0]:
            raise ValueError("the Hadamard ensemble has at most n' rows")
        return srht_entries(seed, stream_id, rows, cols, n) / np.sqrt(float(m))
    return phi_entries(ens, seed, stream_id, rows, cols) / np.sqrt(float(m))
