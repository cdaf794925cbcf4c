"""CPU oracle for the measurement-and-recovery path (test infrastructure only).

Plain NumPy, fp64, one function per operation, written from the paper's
definitions (Secs. 3, 6, 7, 8, 9).  It shares no code with the HIP library and
must never be imported by the product path: only the test-suite, the smoke
check and the benchmark's CPU-baseline leg call it.

Pin status of each function (what ties it to something other than itself):

* philox4x32_10      -- published known-answer vectors of the generator.
* phi_entries        -- statistical tests (moments, unit column norms, nested
                        rows); the (seed, stream, row, col) -> counter mapping
                        is this project's own convention: parity unpinned by
                        any external vector beyond the generator itself.
* phi_matrix (SRHT)  -- equals R H D written out with a library Hadamard matrix, the row map is a
                        bijection, Phi Phi^T = (n/m) I when n is a power of two, a textbook fast
                        Walsh-Hadamard transform gives the same sketch, norm preservation in
                        expectation; the (seed, stream) -> signs and rows mapping is this
                        project's own convention (parity unpinned beyond the generator).
* sketch             -- equals an explicit dense matrix-vector product;
                        linearity; norm preservation in expectation.
* block_omp          -- brute force over all supports, closed forms for
                        orthonormal dictionaries, the incoherence guarantee of
                        Prop. 1, exactness in the noiseless case (Thm. 1),
                        sample-complexity shape of Thm. 2, library lstsq.
* block_iht          -- closed form for orthonormal dictionaries (one step is exact), fixed
                        point at the planted solution, exact recovery of well-separated
                        planted supports, brute force on tiny instances, step length
                        against an explicit line search, library lstsq for the refit.
* incremental_block_omp -- swaps = k is block_omp itself, swaps = 0 is library lstsq on the
                        previous support, brute force over every support within the drift
                        budget (orthonormal dictionaries: exact), closed-form ridge for the
                        regularised refit, the gamma -> infinity limit, planted drift, and
                        the measurement saving of the incremental proposition (Sec. 10).
* support_drift      -- hand-computed examples of D_t (Sec. 15).
* block_ffn          -- dense SwiGLU via an independent formulation, masked
                        dense identity (Sec. 3), additivity over supports.
* head_attn          -- full softmax attention, L=1, uniform-key closed forms.
* softmax_entropy / uds_budget -- uniform, two-point and peaked distributions in closed form,
                        a library routine for the entropy, hand-computed budgets and clipping.
* top_k / joint      -- full sort, permutation invariance, k=n.
* joint_select_coupled -- pooled sketch = sketch of the pooled usage (linearity), k_tok = n
                        reduces to the mean over all tokens, planted prompts where the kept
                        tokens share one support and the dropped ones do not.
* c_twin (plain C)   -- the decode-step functions (generator, operator entries, sketch, effective
                        matrix with one atom per unit, block_omp, block_ffn, head_attn) written
                        again as C loops for the CPU-baseline timing; pinned by the generator's
                        known-answer vectors, exhaustive search over supports, the masked dense
                        identity, full softmax attention, library least squares, and agreement
                        with the NumPy functions above to rounding.  No parity test of the HIP
                        path depends on it.
"""
from .philox import philox4x32_10
from .operator import phi_entries, phi_matrix, srht_rows, srht_order, GAUSS, RADEMACHER, SRHT
from .sketch import sketch
from .recover import effective_matrix, block_omp
from .iht import block_iht
from .incremental import incremental_block_omp, support_drift
from .ffn import block_ffn
from .attn import head_attn
from .controller import softmax_entropy, uds_budget
from .joint import top_k_indices, token_proxy, joint_select, joint_select_coupled

__all__ = [
    "philox4x32_10", "phi_entries", "phi_matrix", "srht_rows", "srht_order", "GAUSS", "RADEMACHER", "SRHT",
    "sketch", "effective_matrix", "block_omp", "block_iht", "incremental_block_omp", "support_drift", "block_ffn", "head_attn",
    "softmax_entropy", "uds_budget", "top_k_indices", "token_proxy", "joint_select", "joint_select_coupled",
]
