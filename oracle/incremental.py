"""Warm-started (incremental) structured recovery (oracle, fp64).

The paper's token-adaptive loop (Sec. 5) regularises the per-token recovery towards
the previous token's solution, Omega_temp = gamma ||alpha_t - alpha_{t-1}||^2 (a penalty
on the change of support is allowed instead), and argues (Sec. 10, proposition on incremental
token-adaptive recovery) that when the support drifts by Delta_t = |S_t ^ S_{t-1}|
units only the changed part has to be identified, from about
Delta_t log(e G / Delta_t) measurements.  It prints no procedure.  The one taken
here is a backward/forward exchange around the previous support, with `swaps` as the
drift budget (swaps units may leave and the same number enter, so up to
Delta_t = 2*swaps):

    1. refit on the previous support S_prev with the temporal regulariser:
           alpha1 = argmin_a ||y - M_S a||^2 + gamma ||a - alpha_prev||^2
       (gamma = 0, or no previous coefficients: the plain least-squares refit);
    2. backward step: drop the `swaps` units of S_prev with the least energy
       (same unit energy as the thresholding solver: the unit's coefficients scaled
       by their atoms' norms when the greedy score is normalised, raw otherwise);
       among equal energies the larger unit index is dropped first;
    3. forward step: `swaps` rounds of the greedy rule of block_omp (score the
       unselected units on the residual of the least-squares fit of the current
       units, take the best, ties -> smallest index, refit, new residual);
    4. plain least-squares refit on the final support.

swaps = k drops everything and is block_omp itself; swaps = 0 keeps S_prev and only
refits.  The support-drift metric of Sec. 15, D_t = |S_t ^ S_{t-1}| / |S_t u S_{t-1}|,
is `support_drift`.
"""
import numpy as np
from .recover import _least_squares


def support_drift(s_now, s_prev):
    """D_t = |S_t symmetric-difference S_{t-1}| / |S_t union S_{t-1}| (0 for two empty sets)."""
    a, b = set(int(v) for v in s_now), set(int(v) for v in s_prev)
    union = a | b
    return len(a ^ b) / len(union) if union else 0.0


def _cols(units, rb):
    return np.concatenate([np.arange(g * rb, (g + 1) * rb) for g in units]) if len(units) else np.zeros(0, dtype=np.int64)


def incremental_block_omp(M, y, G, rb, k, prev_support, swaps, normalised, prev_coef=None, gamma=0.0,
                          prefer=None, slack=0.0):
    """Returns a dict: support (ascending), coef ([k*rb], ascending-support order, plain refit),
    residual, resid_norm, margin (min over the forward rounds of (best - runner_up)/best; 1 when
    swaps == 0), kept / dropped / added (unit lists), coef_step1 (the regularised refit on
    prev_support, in prev_support order), drop_margin (relative energy gap between the last unit
    dropped and the weakest unit kept; 1 when nothing or everything is dropped).

    prev_support: k distinct units in any order; prev_coef: [k*rb] in the order of prev_support.

    prefer, slack: as in block_omp, for checking a support selected elsewhere: a unit of `prefer`
    is ranked as if its energy (backward step) or score (forward step) were (1 + slack) times
    larger.  Defaults: the plain rule.
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
    if not (0 <= swaps <= k):
        raise ValueError("swaps out of range")
    prev = [int(g) for g in prev_support]
    if len(prev) != k or len(set(prev)) != k or min(prev) < 0 or max(prev) >= G:
        raise ValueError("prev_support must hold k distinct units")
    if gamma < 0.0:
        raise ValueError("gamma must be >= 0")
    norms = np.linalg.norm(M, axis=0)
    weights = norms if normalised else np.ones(G * rb)
    boost = np.ones(G)
    if prefer is not None:
        boost[[int(g) for g in prefer]] = 1.0 + slack

    # 1. temporal-regularised refit on the previous support (normal equations of the stacked system)
    cols = _cols(prev, rb)
    A = M[:, cols]
    if prev_coef is not None and gamma > 0.0:
        ap = np.asarray(prev_coef, dtype=np.float64).reshape(k * rb)
        A_aug = np.vstack([A, np.sqrt(gamma) * np.eye(k * rb)])
        y_aug = np.concatenate([y, np.sqrt(gamma) * ap])
        alpha1 = _least_squares(A_aug, y_aug)
    else:
        alpha1 = _least_squares(A, y)

    # 2. backward step
    energy = ((alpha1 * weights[cols]) ** 2).reshape(k, rb).sum(axis=1)
    order = sorted(range(k), key=lambda i: (energy[i] * boost[prev[i]], -prev[i]))      # first = dropped first
    e_sorted = [energy[i] for i in order]
    if 0 < swaps < k and e_sorted[swaps] > 0.0:
        drop_margin = float((e_sorted[swaps] - e_sorted[swaps - 1]) / e_sorted[swaps])
    else:
        drop_margin = 1.0 if swaps in (0, k) else 0.0
    dropped = [prev[i] for i in order[:swaps]]
    chosen = [prev[i] for i in order[swaps:]]
    kept = list(chosen)

    # 3. forward step: greedy rounds from the kept units
    bases = None
    if normalised:
        bases = [np.linalg.qr(M[:, g * rb:(g + 1) * rb])[0] for g in range(G)]
    margin = 1.0
    added = []
    for _ in range(swaps):
        if chosen:
            cc = _cols(chosen, rb)
            r = y - M[:, cc] @ _least_squares(M[:, cc], y)
        else:
            r = y.copy()
        score = np.full(G, -np.inf)
        for g in range(G):
            if g in chosen:
                continue
            c = bases[g].T @ r if normalised else M[:, g * rb:(g + 1) * rb].T @ r
            score[g] = float(c @ c)
        best = int(np.argmax(score * boost))
        s1 = score[best]
        rest = np.delete(score, best)
        s2 = float(rest.max()) if rest.size and np.isfinite(rest.max()) else 0.0
        margin = min(margin, (s1 - s2) / s1) if s1 > 0.0 else 0.0
        chosen.append(best)
        added.append(best)

    # 4. final refit
    support = sorted(chosen)
    cc = _cols(support, rb)
    coef = _least_squares(M[:, cc], y)
    r = y - M[:, cc] @ coef
    return {
        "support": np.array(support, dtype=np.int32),
        "coef": coef,
        "residual": r,
        "resid_norm": float(np.linalg.norm(r)),
        "margin": float(margin),
        "kept": kept,
        "dropped": dropped,
        "added": added,
        "coef_step1": alpha1,
        "drop_margin": drop_margin,
    }
