"""Structured sparse recovery: block orthogonal matching pursuit (oracle, fp64).

The paper models the usage vector as u ~ Psi alpha with one group of
coefficients per structured unit (Sec. 3), senses it with M = A Psi (Sec. 9),
and lists greedy pursuit restricted to a dictionary of admissible supports
among the per-token solvers (Sec. 8); the support is then projected onto the
admissible family (Sec. 3, Sec. 7).  Here the admissible family is "exactly k
units", and the greedy rule is the classical one:

    repeat k times
        score every unselected unit by the energy of the residual in the
            unit's column space (or, for an identity dictionary, by the raw
            block energy of the correlation M_g^T r),
        pick the best unit (ties -> smallest index),
        refit all selected coefficients by least squares,
        recompute the residual.

The refit uses a Householder QR (numpy.linalg.qr) and a triangular solve.
"""
import numpy as np
from .operator import phi_matrix


def effective_matrix(ens, seed, stream_id, m, n, G, b, rb, psi=None):
    """M = Phi Psi for a block-diagonal dictionary.

    psi: [G, b, rb] (unit g maps its rb coefficients onto its b channels), or
    None for the identity dictionary (rb == b).  Returns M as [m, G*rb] with
    unit g owning columns g*rb .. g*rb+rb-1.
    """
    if n != G * b:
        raise ValueError("n must equal G*b")
    if psi is None:
        if rb != b:
            raise ValueError("identity dictionary needs rb == b")
        return phi_matrix(ens, seed, stream_id, m, n)
    psi = np.asarray(psi, dtype=np.float64).reshape(G, b, rb)
    M = np.empty((m, G * rb), dtype=np.float64)
    for g in range(G):
        phi_g = phi_matrix(ens, seed, stream_id, m, n, g * b, b)     # [m, b]
        M[:, g * rb:(g + 1) * rb] = phi_g @ psi[g]
    return M


def _least_squares(A, y):
    q, r = np.linalg.qr(A)                      # Householder, reduced
    rhs = q.T @ y
    coef = np.zeros(A.shape[1])
    for i in range(A.shape[1] - 1, -1, -1):     # back substitution
        coef[i] = (rhs[i] - r[i, i + 1:] @ coef[i + 1:]) / r[i, i]
    return coef


def block_omp(M, y, G, rb, k, normalised, prefer=None, slack=0.0):
    """Greedy recovery of k units from y ~ M alpha.

    normalised=True : score_g = || Q_g^T r ||^2, Q_g an orthonormal basis of
                      the unit's columns (for rb == 1: (m_g^T r)^2 / ||m_g||^2,
                      the normalised-column correlation of Sec. 9).
    normalised=False: score_g = || M_g^T r ||^2 (raw block energy).

    prefer, slack: for checking a support that somebody else selected.  Near
    ties have several correct greedy choices; with prefer = that support and a
    small slack, a unit of `prefer` is taken whenever its score is within a
    factor 1/(1+slack) of the best one.  The other support is a valid greedy
    path up to that slack exactly when this call returns it.  The defaults
    (no preference) are the rule stated above.

    Returns a dict: support (ascending), order (selection order), coef
    ([k*rb], in ascending-support order), residual (vector), resid_norm,
    margin = min over rounds of (best - runner_up) / best.
    """
    M = np.asarray(M, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    m = M.shape[0]
    if M.shape[1] != G * rb:
        raise ValueError("M has the wrong number of columns")
    if not (1 <= k <= G):
        raise ValueError("k out of range")
    if k * rb >= m:
        raise ValueError("ill-posed: k*rb must be < m")
    bases = None
    if normalised:
        bases = [np.linalg.qr(M[:, g * rb:(g + 1) * rb])[0] for g in range(G)]
    boost = np.ones(G)
    if prefer is not None:
        boost[[int(g) for g in prefer]] = 1.0 + slack
    chosen = []
    r = y.copy()
    margin = 1.0
    for _ in range(k):
        score = np.full(G, -np.inf)
        for g in range(G):
            if g in chosen:
                continue
            if normalised:
                c = bases[g].T @ r
            else:
                c = M[:, g * rb:(g + 1) * rb].T @ r
            score[g] = float(c @ c)
        best = int(np.argmax(score * boost))     # first maximum = smallest index
        s1 = score[best]
        rest = np.delete(score, best)
        s2 = float(rest.max()) if rest.size and np.isfinite(rest.max()) else 0.0
        margin = min(margin, (s1 - s2) / s1) if s1 > 0.0 else 0.0
        chosen.append(best)
        cols = np.concatenate([np.arange(g * rb, (g + 1) * rb) for g in chosen])
        coef_sel = _least_squares(M[:, cols], y)
        r = y - M[:, cols] @ coef_sel
    support = sorted(chosen)
    cols = np.concatenate([np.arange(g * rb, (g + 1) * rb) for g in support])
    coef = _least_squares(M[:, cols], y)
    r = y - M[:, cols] @ coef
    return {
        "support": np.array(support, dtype=np.int32),
        "order": np.array(chosen, dtype=np.int32),
        "coef": coef,
        "residual": r,
        "resid_norm": float(np.linalg.norm(r)),
        "margin": float(margin),
    }
