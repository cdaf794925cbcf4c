"""Joint prompt-token and channel-block selection (oracle, fp64).

Sec. 6 couples a token-retention vector r with the unit support.  The paper
gives the objective but no procedure; the procedure used here is the simplest
one consistent with it: tokens are kept by one-step thresholding of the
back-projected token sketch (greedy pursuit is impossible because more tokens
are kept than there are measurements), and the channel support comes from block
OMP on the channel sketch.
"""
import numpy as np
from .operator import phi_matrix
from .recover import block_omp


def top_k_indices(scores, k):
    """Indices of the k largest scores (signed), ties -> lower index, returned
    in ascending index order."""
    scores = np.asarray(scores, dtype=np.float64)
    order = sorted(range(scores.size), key=lambda i: (-scores[i], i))
    return np.array(sorted(order[:k]), dtype=np.int32)


def token_proxy(ens, seed, stream_id, m, n, y_tok):
    """p = Phi^T y: the matched-filter estimate of per-token saliency."""
    phi = phi_matrix(ens, seed, stream_id, m, n)
    return phi.T @ np.asarray(y_tok, dtype=np.float64)


def joint_select(tok_op, y_tok, k_tok, M_ch, y_ch, G, rb, k_ch, normalised):
    """tok_op = (ens, seed, stream_id, m, n).  Returns (tokens, recovery dict, proxy)."""
    p = token_proxy(*tok_op, y_tok)
    tokens = top_k_indices(p, k_tok)
    rec = block_omp(M_ch, y_ch, G, rb, k_ch, normalised)
    return tokens, rec, p
