"""Joint prompt-token and channel-block selection (oracle, fp64).

Sec. 6 couples a token-retention vector r with the unit support.  The paper
gives the objective but no procedure; the procedure used here is the simplest
one consistent with it: tokens are kept by one-step thresholding of the
back-projected token sketch (greedy pursuit is impossible because more tokens
are kept than there are measurements), and the channel support comes from block
OMP on the channel sketch.

`joint_select` keeps the two decisions independent (the "sequential" arm of the
ablation list in Sec. 15).  `joint_select_coupled` is the smallest procedure in
which the retained tokens change the measurement the support is recovered from,
as the constraint z_t = A_t(r) Psi(r) alpha_t of Sec. 6 demands: the channel sketch
is pooled over the retained tokens only,

    ybar(r) = mean_{t in r} y_t,      y_t = Phi_ch z_t,

which by linearity of the sketch is the sketch of the retained tokens' mean usage,
and the support is recovered from ybar(r).
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


def joint_select_coupled(tok_op, y_tok, k_tok, M_ch, Y_ch, G, rb, k_ch, normalised):
    """Y_ch: [n_tok, m] per-token channel sketches.  Returns (tokens, ybar, recovery dict, proxy):
    tokens as in joint_select, ybar = mean of the retained tokens' sketches, recovery = block_omp(ybar)."""
    Y_ch = np.asarray(Y_ch, dtype=np.float64)
    p = token_proxy(*tok_op, y_tok)
    tokens = top_k_indices(p, k_tok)
    ybar = np.zeros(Y_ch.shape[1])
    for t in tokens:
        ybar += Y_ch[int(t)]
    ybar /= len(tokens)
    rec = block_omp(M_ch, ybar, G, rb, k_ch, normalised)
    return tokens, ybar, rec, p
