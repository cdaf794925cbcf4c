"""Head-pruned single-query attention over a key/value cache (oracle, fp64).

Heads are the structured units here (Sec. 3, Sec. 7): a kept head computes
ordinary scaled-dot-product attention of its query against all cached
positions; a pruned head is masked off and outputs zeros.
"""
import numpy as np


def head_attn(q, K, V, heads):
    """q: [B, H, dh]; K, V: [B, H, L, dh]; heads: [B, kh] kept head indices.
    Returns out [B, H, dh] (fp64)."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, H, dh = q.shape
    out = np.zeros((B, H, dh), dtype=np.float64)
    for bi in range(B):
        for h in np.asarray(heads)[bi]:
            s = K[bi, h] @ q[bi, h] / np.sqrt(float(dh))      # [L]
            p = np.exp(s - s.max())
            p /= p.sum()
            out[bi, h] = p @ V[bi, h]
    return out
