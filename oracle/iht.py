"""Structured sparse recovery by projected gradient steps: block iterative hard
thresholding (oracle, fp64).

The paper names proximal steps followed by a projection, run for a small fixed
number of iterations, as the second cheap solver next to greedy pursuit (Sec. 8), with the
projection onto the admissible supports of Sec. 7 (here: exactly k units).  The
iteration is the classical normalised hard-thresholding scheme:

    g      = M^T (y - M alpha)                    gradient of the data term
    mu     = ||g_S||^2 / ||M g_S||^2              exact line search on the current support S
                                                  (first step: S = the k units with most gradient energy)
                                                  stop when ||g_S|| <= 1e-3 of its value in the first step:
                                                  alpha is then the least-squares fit on S and the line
                                                  search would divide rounding noise by rounding noise
    p      = alpha + mu g
    S      = the k units with the largest energy of p   (ties -> smaller index)
    alpha  = p restricted to S
    
repeated a fixed number of times, followed by one least-squares refit on the final
support.  Unit energies use the same weighting as the greedy solver: with a
dictionary the unit's entries are scaled by their atoms' norms (rb = 1: (p_g ||m_g||)^2),
with the identity dictionary the raw sum of squares.
"""
import numpy as np


STOP_REL = 1e-3      # the iteration stops once the gradient on the support is this small against its first value


def _unit_energy(v, G, rb, weights):
    e = (v * weights) ** 2
    return e.reshape(G, rb).sum(axis=1)


def _top_units(energy, k, boost=None):
    key = energy if boost is None else energy * boost
    order = sorted(range(energy.size), key=lambda g: (-key[g], g))
    return sorted(order[:k]), order


def block_iht(M, y, G, rb, k, iters, normalised, prefer=None, slack=0.0):
    """Returns a dict like block_omp: support (ascending), coef ([k*rb], ascending-support
    order, after the final refit), residual, resid_norm, margin = relative gap between the
    k-th and (k+1)-th unit energies at the last projection (1 if k == G).

    prefer, slack: as in block_omp, for checking a support selected elsewhere: in every
    projection a unit of `prefer` is ranked as if its energy were (1 + slack) times larger, so
    that near ties at the cut fall towards `prefer`.  Defaults: the plain rule."""
    M = np.asarray(M, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    m, N = M.shape
    if N != G * rb:
        raise ValueError("M has the wrong number of columns")
    if not (1 <= k <= G):
        raise ValueError("k out of range")
    if k * rb >= m:
        raise ValueError("ill-posed: k*rb must be < m")
    if iters < 1:
        raise ValueError("iters must be >= 1")
    weights = np.linalg.norm(M, axis=0) if normalised else np.ones(N)
    boost = None
    if prefer is not None:
        boost = np.ones(G)
        boost[[int(u) for u in prefer]] = 1.0 + slack
    alpha = np.zeros(N)
    support = None
    margin = 1.0
    min_margin = 1.0
    num0 = None
    for _ in range(iters):
        g = M.T @ (y - M @ alpha)
        if support is None:
            e0 = _unit_energy(g, G, rb, weights)
            support, order0 = _top_units(e0, k, boost)
            if k < G and e0[order0[k - 1]] > 0.0:
                min_margin = min(min_margin, (e0[order0[k - 1]] - e0[order0[k]]) / e0[order0[k - 1]])
        cols = np.concatenate([np.arange(u * rb, (u + 1) * rb) for u in support])
        gs = np.zeros(N)
        gs[cols] = g[cols]
        num = float(gs @ gs)
        if num0 is None:
            num0 = num
        elif num <= STOP_REL ** 2 * num0:
            break                                  # converged on this support: support, alpha and margin stand
        den = float(np.sum((M @ gs) ** 2))
        mu = num / den if den > 0.0 else 0.0
        p = alpha + mu * g
        energy = _unit_energy(p, G, rb, weights)
        support, order = _top_units(energy, k, boost)
        if k < G:
            ek, ek1 = energy[order[k - 1]], energy[order[k]]
            margin = (ek - ek1) / ek if ek > 0.0 else 0.0
        else:
            margin = 1.0
        min_margin = min(min_margin, margin)
        cols = np.concatenate([np.arange(u * rb, (u + 1) * rb) for u in support])
        alpha = np.zeros(N)
        alpha[cols] = p[cols]
    cols = np.concatenate([np.arange(u * rb, (u + 1) * rb) for u in support])
    coef, *_ = np.linalg.lstsq(M[:, cols], y, rcond=None)
    r = y - M[:, cols] @ coef
    return {
        "support": np.array(support, dtype=np.int32),
        "coef": coef,
        "residual": r,
        "resid_norm": float(np.linalg.norm(r)),
        "margin": float(margin),
        "min_margin": float(min_margin),     # smallest projection gap over all rounds (for test filtering)
    }
