"""Uncertainty-driven measurement budget (oracle, fp64).

Sec. 8.1 sets the number of measurements of step t from the entropy of the previous
step's predictive distribution,

    H(p)  = - sum_v p(v) log p(v)                       (natural logarithm, 0 log 0 = 0)
    m_t   = clip( floor( m_base (1 + gamma H(p_{t-1})) ), m_min, m_max ).

The distribution is given by its logits: p = softmax(logits).
"""
import math
import numpy as np


def softmax_entropy(logits):
    """Entropy in nats of softmax(logits); logits: [B, V] (or [V]) -> [B] (or scalar)."""
    x = np.asarray(logits, dtype=np.float64)
    single = x.ndim == 1
    x2 = x[None, :] if single else x
    out = np.empty(x2.shape[0])
    for i in range(x2.shape[0]):
        row = x2[i] - np.max(x2[i])
        p = np.exp(row)
        p /= p.sum()
        nz = p > 0.0
        out[i] = -float(np.sum(p[nz] * np.log(p[nz])))
    return float(out[0]) if single else out


def uds_budget(m_base, gamma, entropy, m_min, m_max):
    """m_t = clip(floor(m_base (1 + gamma H)), m_min, m_max)."""
    if m_min > m_max:
        raise ValueError("m_min > m_max")
    return int(min(max(math.floor(m_base * (1.0 + gamma * entropy)), m_min), m_max))
