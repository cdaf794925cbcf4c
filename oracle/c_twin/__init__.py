"""ctypes front of the plain C twin of the decode-step oracle (test infrastructure only).

`build()` compiles cs_oracle.c with gcc (-O2, OpenMP pragmas honoured, nothing else) into a shared
object beside it; the functions below marshal NumPy fp64 arrays and call it.  Same argument
conventions as the NumPy oracle's functions of the same names.  Only tests, the smoke check and the
benchmark's CPU-baseline leg may use it.
"""
import ctypes
import os
import subprocess

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "cs_oracle.c")
LIB = os.path.join(HERE, "libcs_oracle.so")
_lib = None


def build():
    """Compile the twin (every time it is called)."""
    cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Werror", SRC, "-o", LIB, "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode:
        raise RuntimeError("gcc failed:\n" + r.stderr)
    return LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
            build()
        lib = ctypes.CDLL(LIB)
        dp, ip = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)
        u32p = ctypes.POINTER(ctypes.c_uint32)
        i, u64, u32 = ctypes.c_int, ctypes.c_uint64, ctypes.c_uint32
        lib.cso_set_threads.argtypes = [i]
        lib.cso_set_threads.restype = i
        lib.cso_philox4x32_10.argtypes = [u32p, u32p, u32p]
        lib.cso_philox4x32_10.restype = None
        lib.cso_phi_entry.argtypes = [i, u64, u32, u32, u32]
        lib.cso_phi_entry.restype = ctypes.c_double
        lib.cso_sketch.argtypes = [i, u64, u32, i, i, dp, i, dp]
        lib.cso_sketch.restype = None
        lib.cso_effective_matrix.argtypes = [i, u64, u32, i, i, i, dp, dp]
        lib.cso_effective_matrix.restype = None
        lib.cso_block_omp.argtypes = [dp, i, i, dp, i, i, i, ip, dp, dp, dp]
        lib.cso_block_omp.restype = i
        lib.cso_block_ffn.argtypes = [dp, dp, dp, i, i, i, dp, i, ip, i, i, dp]
        lib.cso_block_ffn.restype = None
        lib.cso_head_attn.argtypes = [dp, dp, dp, i, i, i, i, ip, i, dp]
        lib.cso_head_attn.restype = None
        _lib = lib
    return _lib


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _i(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def set_threads(n):
    """Threads of the twin's parallel loops from now on (n < 1: all the runtime offers); returns the count."""
    return int(_load().cso_set_threads(int(n)))


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    ctr = (ctypes.c_uint32 * 4)(c0, c1, c2, c3)
    key = (ctypes.c_uint32 * 2)(k0, k1)
    out = (ctypes.c_uint32 * 4)()
    _load().cso_philox4x32_10(ctr, key, out)
    return tuple(int(v) for v in out)


def phi_entry(ens, seed, stream_id, row, col):
    return float(_load().cso_phi_entry(ens, seed, stream_id, row, col))


def sketch(ens, seed, stream_id, m, z):
    z, zp = _d(z)
    single = z.ndim == 1
    B, n = (1, z.shape[0]) if single else z.shape
    y = np.empty((B, m), dtype=np.float64)
    _load().cso_sketch(ens, seed, stream_id, m, n, zp, B, y.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return y[0] if single else y


def effective_matrix(ens, seed, stream_id, m, n, G, b, rb, psi=None):
    """One atom per unit only: rb == 1 with a dictionary [G, b, 1], or the identity dictionary with b == 1."""
    if n != G * b or rb != 1 or (psi is None and b != 1):
        raise ValueError("the C twin covers one atom per unit")
    M = np.empty((m, G), dtype=np.float64)
    if psi is None:
        pp = None
    else:
        psi, pp = _d(np.asarray(psi, dtype=np.float64).reshape(G, b))
    _load().cso_effective_matrix(ens, seed, stream_id, m, G, b, pp, M.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return M


def block_omp(M, Y, G, k, normalised):
    """Y: [B, m] (or [m]).  Returns (support [B, k] ascending, coef [B, k], resid_norm [B], margin [B])."""
    M, Mp = _d(M)
    Y, Yp = _d(Y)
    single = Y.ndim == 1
    B = 1 if single else Y.shape[0]
    m = M.shape[0]
    sup = np.empty((B, k), dtype=np.int32)
    coef = np.empty((B, k), dtype=np.float64)
    res = np.empty((B,), dtype=np.float64)
    mar = np.empty((B,), dtype=np.float64)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = _load().cso_block_omp(Mp, m, G, Yp, B, k, 1 if normalised else 0, sup.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                               coef.ctypes.data_as(dp), res.ctypes.data_as(dp), mar.ctypes.data_as(dp))
    if rc:
        raise ValueError("k out of range or ill-posed (k must be < m)")
    return (sup[0], coef[0], res[0], mar[0]) if single else (sup, coef, res, mar)


def block_ffn(Wg, Wu, Wd, x, support):
    Wg, gp = _d(Wg)
    Wu, up = _d(Wu)
    Wd, dp_ = _d(Wd)
    x, xp = _d(x)
    sup, sp = _i(support)
    G, b, d = Wg.shape
    T = x.shape[0]
    shared = sup.ndim == 1
    k = sup.shape[-1]
    out = np.empty((T, d), dtype=np.float64)
    _load().cso_block_ffn(gp, up, dp_, G, b, d, xp, T, sp, k, 1 if shared else 0, out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return out


def head_attn(q, K, V, heads):
    q, qp = _d(q)
    K, kp = _d(K)
    V, vp = _d(V)
    heads, hp = _i(heads)
    B, H, dh = q.shape
    L = K.shape[2]
    out = np.empty((B, H, dh), dtype=np.float64)
    _load().cso_head_attn(qp, kp, vp, B, H, L, dh, hp, heads.shape[1], out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return out
