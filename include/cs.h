/*
 * cs.h -- C ABI of the measurement-and-recovery library (MI355X / gfx950).
 *
 * The library implements the online phase of compressed-sensing-guided sparse
 * execution (paper Sec. 12, "online phase"): sketch the latent usage vector
 * with a random operator, recover the active structured units by block
 * orthogonal matching pursuit, and execute only those units (block-sparse
 * gated FFN, head-pruned attention), plus joint token/unit selection (Sec. 6).
 *
 * Conventions common to every call
 *  - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *    never frees or keeps it beyond the stream order of the call.
 *  - Work is enqueued on the context's HIP stream; no call synchronises the
 *    device.  Results are valid once the caller has synchronised that stream.
 *  - Device pointers must be 16-byte aligned (CS_EALIGN otherwise).
 *  - Errors are reported by return code, never by exception; arguments are
 *    checked on the host before anything is launched.  cs_last_error() gives
 *    a message for the last failing call on the context.
 *  - The context owns a scratch buffer (sized at cs_create) and a cache of
 *    per-operator plans.  The five hot calls allocate nothing once the plan
 *    they need exists (see cs_plan).
 */
#ifndef CS_H_
#define CS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cs_ctx cs_ctx;

typedef enum {
    CS_OK = 0,
    CS_EINVAL = -1,     /* bad argument (range, shape, null pointer, unsupported combination) */
    CS_EALIGN = -2,     /* a device pointer is not 16-byte aligned */
    CS_EILLPOSED = -3,  /* recovery with k*rb >= m: the refit would be under-determined */
    CS_ENOMEM = -4,     /* scratch buffer too small, or a device allocation failed */
    CS_EHIP = -5        /* a HIP runtime call failed; text in cs_last_error */
} cs_status;

typedef enum { CS_GAUSS = 0, CS_RADEMACHER = 1, CS_SRHT = 2 } cs_ensemble;
typedef enum { CS_F32 = 0, CS_BF16 = 1 } cs_dtype;

/*
 * Measurement operator Phi (the paper's A_t, Sec. 3 and Sec. 8): an m x n random
 * matrix from a subgaussian ensemble.  It is never stored: entry (row, col) is a
 * pure function of (seed, stream_id, row, col) through the Philox4x32-10 counter
 * generator:
 *   key = (seed & 0xffffffff, seed >> 32), counter = (col / cpc, row, stream_id, ens)
 *   Rademacher: cpc = 128; column c reads bit (c % 32) of output word ((c % 128) / 32);
 *               bit 0 -> +1, bit 1 -> -1.
 *   Gaussian:   cpc = 4; p = (c % 4) / 2; u1 = (w[2p]+1)/2^32, u2 = (w[2p+1]+1)/2^32;
 *               even columns sqrt(-2 ln u1) cos(2 pi u2), odd columns ... sin(2 pi u2).
 *   Subsampled randomised Hadamard (CS_SRHT; Sec. 8 names it for implementation efficiency):
 *               Phi = (1/sqrt(m)) R H D on the first n columns, H the Walsh-Hadamard matrix of
 *               order n' = 2^b, the smallest power of two >= max(n, 2), H[r][c] =
 *               (-1)^popcount(r & c); d_c = Rademacher bit of column c under counter
 *               (c / 128, 0, stream_id, 2); measurement i reads row r_i = perm(i), with w the
 *               output of counter (0, 1, stream_id, 2): x = (i (w0|1) + w1) mod n';
 *               x ^= x >> ceil(b/2); x = (x (w2|1) + w3) mod n'; x ^= x >> ceil(b/2).
 *               Needs m <= n'; cs_sketch evaluates it by a fast transform and needs n' <= 32768.
 *   Phi[row][col] = entry / sqrt(m).
 * Rows do not depend on m, so a change of the measurement budget (Sec. 8.1) only
 * adds or removes rows and rescales.
 */
typedef struct {
    int32_t  ens;        /* cs_ensemble */
    uint64_t seed;
    uint32_t stream_id;  /* selects one operator of a bank (layer, kind) */
    int32_t  m;          /* rows = number of measurements */
    int32_t  n;          /* columns = length of the usage vector */
} cs_op;

/*
 * Structured dictionary Psi (Sec. 3): block diagonal, unit g maps rb coefficients
 * onto its b contiguous channels.  psi is a device array float[G][b][rb] whose
 * columns within a unit are linearly independent, or NULL for the identity
 * dictionary (then rb must equal b).  The effective sensing matrix is
 * M = Phi Psi (Sec. 9), unit g owning columns g*rb .. g*rb+rb-1.
 */
typedef struct {
    const float* psi;
    int32_t G, b, rb;
} cs_dict;

/* Create a context bound to `device` and to `hip_stream` (a hipStream_t, may be
 * NULL for the default stream).  scratch_bytes of device memory are allocated
 * once and reused by every call (0 selects 64 MiB).  Calls on one context must
 * not overlap in time.  Returns CS_EHIP / CS_ENOMEM on failure. */
cs_status cs_create(cs_ctx** out, int device, void* hip_stream, size_t scratch_bytes);
void cs_destroy(cs_ctx* ctx);
const char* cs_last_error(const cs_ctx* ctx);
/* Rebind the context to another stream (no synchronisation is performed). */
cs_status cs_set_stream(cs_ctx* ctx, void* hip_stream);

/*
 * What the caller knows about the union of the per-row supports of the cs_block_ffn calls to come
 * (token-adaptive decode, Sec. 5: rows of a batch may share most of their units or none).  With 2 to 64 rows
 * the first weights are requested at kernel entry, before the supports have been read, for the blocks a
 * dense union implies; if the union turns out sparse those loads are wasted (results are the same).
 *   CS_UNION_AUTO   (default) dense is assumed when the rows list at least 2 G entries (4 G above 16 rows)
 *   CS_UNION_DENSE  the rows' supports are independent enough to cover nearly all G units
 *   CS_UNION_SPARSE the rows share most of their units: wait for the list
 * Anything else is CS_EINVAL.  The hint stays until it is set again.
 */
enum { CS_UNION_AUTO = 0, CS_UNION_DENSE = 1, CS_UNION_SPARSE = 2 };
cs_status cs_set_union_hint(cs_ctx* ctx, int hint);

/*
 * Build and cache the plan of (op, dict): the effective matrix M = Phi Psi, its
 * column Gram matrix and the per-unit score weights (Sec. 9: M_t = A_t Psi, and
 * the normalised columns used in the coherence definition).  Allocates device
 * memory the context keeps until cs_destroy.  cs_recover_support and
 * cs_joint_select call it implicitly on first use of an (op, dict) pair; calling
 * it beforehand keeps allocation out of the hot loop.  The content of dict->psi
 * is read at plan time only.
 */
cs_status cs_plan(cs_ctx* ctx, const cs_op* op, const cs_dict* dict);

/*
 * Plans are found again by the fields of `op` and by dict->psi, G, b, rb: the dictionary is identified by
 * its ADDRESS, not by its content, and it is read at plan time only.  A caller that frees a dictionary,
 * or overwrites it, must drop the plans built from it before the same address is used for other content;
 * otherwise a later call with that address would silently run on the old plan.  cs_plan_drop waits for
 * the context's stream, frees the plan's device memory (and every multi-operator table that lists it) and
 * forgets it; dropping a pair that has no plan is not an error.  The next use builds a fresh plan.
 */
cs_status cs_plan_drop(cs_ctx* ctx, const cs_op* op, const cs_dict* dict);

/*
 * y = Phi z (measurement equation, Sec. 3 / Sec. 8).
 *   z: float[B][n] in,  y: float[B][m] out.  B >= 0 (B == 0 is a no-op).
 */
cs_status cs_sketch(cs_ctx* ctx, const cs_op* op, const float* z, int B, float* y);

/*
 * cs_sketch for several operators in one launch: y[j] = Phi_j z[j] (Sec. 3 / Sec. 8; Sec. 5: the
 * sketches of a step are only needed by the next step, so the usage vectors of several layers can be
 * kept and measured together).  z: float[n_ops][B][n] in, y: float[n_ops][B][m] out.  All operators
 * must agree in ensemble, m and n; they differ in seed and stream_id.  ops is a host array of n_ops
 * entries, n_ops >= 1.  Each sketch is the same sum of the same exactly representable products as in
 * cs_sketch; large Rademacher launches add them in another order (matrix cores), so the two calls
 * agree to fp32 rounding, bit for bit only on the smaller launches.  Nothing is allocated.
 */
cs_status cs_sketch_multi(cs_ctx* ctx, int n_ops, const cs_op* ops, const float* z, int B, float* y);

/*
 * Structured sparse recovery by block orthogonal matching pursuit over the
 * dictionary's units (Sec. 8 lists greedy pursuit restricted to a dictionary of
 * admissible supports among the per-token solvers; support projection of Sec. 3
 * and Sec. 7 with the admissible family "exactly k units").  For each of the B sketches:
 *   k rounds of { score every unselected unit; take the best (ties -> smaller
 *   index); least-squares refit of all selected coefficients; new residual }.
 * Score of unit g: with a dictionary, the energy of the residual in the unit's
 * column space (for rb == 1 the squared normalised correlation of Sec. 9);
 * with the identity dictionary, the raw block energy ||M_g^T r||^2.
 *   y:          float[B][m] in
 *   support:    int32[B][k] out, ascending unit indices
 *   coef:       float[B][k*rb] out or NULL, coefficients in ascending-unit order
 *   resid_norm: float[B] out or NULL, ||y - M_S coef||_2
 *   margin:     float[B] out or NULL, min over rounds of (best - runner_up)/best;
 *               a small margin means another support was nearly as good
 * Requires 1 <= k <= G, op->n == G*b, k*rb < m (else CS_EILLPOSED).
 * A non-finite sketch or a rank-deficient selection does not abort the call:
 * that problem reports resid_norm = NaN and margin = 0 (the hook for reverting
 * to a denser support, Sec. 12), and its support is still k distinct units.
 */
cs_status cs_recover_support(cs_ctx* ctx, const cs_op* op, const cs_dict* dict, int k,
                             const float* y, int B,
                             int32_t* support, float* coef, float* resid_norm, float* margin);

/*
 * cs_recover_support for several operators in one launch (Sec. 5: the sketch of step t gives the
 * support that the next step executes, so the recoveries of all layers of a step are independent
 * of each other and can be solved together).  Operator j, with dictionary j, serves sketches
 * y[j][0..B) and writes support[j][..], coef[j][..], resid_norm[j][..], margin[j][..]; every
 * array is laid out [n_ops][B][...].  All operators must agree in m and n and all dictionaries in
 * G, b, rb and in having psi or not; the arithmetic per sketch is exactly that of
 * cs_recover_support.  ops and dicts are host arrays of n_ops entries.  The first call with a
 * given list of operators allocates a small device table (like cs_plan); later calls allocate
 * nothing.
 */
cs_status cs_recover_support_multi(cs_ctx* ctx, int n_ops, const cs_op* ops, const cs_dict* dicts, int k,
                                   const float* y, int B,
                                   int32_t* support, float* coef, float* resid_norm, float* margin);

/*
 * Structured sparse recovery by block iterative hard thresholding: the second cheap
 * solver the paper names (Sec. 8: proximal steps followed by a projection, run for a
 * small fixed number of iterations), with the projection onto exactly k units (Sec. 7).
 * `iters` rounds of { g = M^T (y - M alpha); mu = ||g_S||^2 / ||M g_S||^2 on the
 * current support S (first round: the k units with most gradient energy);
 * p = alpha + mu g; S = the k units with the largest energy of p (ties -> smaller
 * index); alpha = p on S }, then one least-squares refit on the final support.
 * Unit energy: (p_g ||m_g||)^2 with a dictionary, p_g^2 with the identity dictionary.
 * Arguments and outputs as cs_recover_support; margin is the relative gap between the
 * k-th and (k+1)-th unit energies at the last projection (1 if k == G).
 * Supported: one atom per unit (rb == 1), k <= 64, G <= 512 (CS_EINVAL otherwise).
 */
cs_status cs_recover_support_iht(cs_ctx* ctx, const cs_op* op, const cs_dict* dict, int k, int iters,
                                 const float* y, int B,
                                 int32_t* support, float* coef, float* resid_norm, float* margin);

/*
 * Warm-started (incremental) recovery: the previous token's support is corrected instead
 * of being recovered from nothing (Sec. 5: temporal regulariser
 * gamma ||alpha_t - alpha_{t-1}||^2 and incremental support updates; Sec. 10, proposition
 * on incremental token-adaptive recovery: a drift of Delta units costs about
 * Delta log(eG/Delta) measurements).  Per sketch:
 *   1. alpha1 = argmin ||y - M_S a||^2 + gamma ||a - alpha_prev||^2 on S = prev_support
 *      (plain least squares when prev_coef is NULL or gamma == 0);
 *   2. the `swaps` units of S with the least energy (alpha1_g ||m_g||)^2 (identity
 *      dictionary: alpha1_g^2) leave, among equal energies the larger index first;
 *   3. `swaps` greedy rounds of cs_recover_support's rule, started from the kept units,
 *      bring the support back to k units;
 *   4. least-squares refit on the final support.
 * swaps == k is cs_recover_support itself; swaps == 0 only refits on prev_support.
 *   prev_support: device int32 [B][k], k distinct units per row in any order
 *   prev_coef:    device float [B][k] in the order of prev_support, or NULL
 *   gamma:        >= 0
 *   swaps:        0 .. k, the drift budget (up to 2*swaps units of symmetric difference)
 *   support, coef, resid_norm: as cs_recover_support; support/coef may alias
 *                 prev_support/prev_coef (a row is read completely before it is written)
 *   margin:       min over the greedy rounds of (best - runner_up)/best; 1 if swaps == 0
 * A row whose prev_support is out of range or repeats a unit, or whose sketch is not
 * finite, does not abort the call: it reports support = -1 in every slot, coef = 0,
 * resid_norm = NaN and margin = 0.
 * Supported: one atom per unit (rb == 1), k <= 64, G <= 512 (CS_EINVAL otherwise).
 */
cs_status cs_recover_support_inc(cs_ctx* ctx, const cs_op* op, const cs_dict* dict, int k,
                                 const float* y, int B,
                                 const int32_t* prev_support, const float* prev_coef, float gamma, int swaps,
                                 int32_t* support, float* coef, float* resid_norm, float* margin);

/*
 * The same exchange (gamma = 0) with state carried from token to token, so that the cost of a
 * token follows its drift and not the size of the support (Sec. 5: the loop runs once per token;
 * Sec. 10, proposition on incremental token-adaptive recovery: only the changed part has to be
 * identified).  Results are those of cs_recover_support_inc with prev_coef == NULL: what differs is
 * how the least-squares fits are solved.  A token leaves the inverse of the Gram matrix of its
 * support behind; the next token fits on that support with one k x k product, removes a unit or
 * adds one with one rank-one correction of the inverse, and no factorisation is computed.
 *   state: device, caller-owned, [B][cs_inc_state_words(k)] 32-bit words, 16-byte aligned; row i
 *          belongs to sketch i of every call of the sequence.  Zero-fill it before the first call
 *          (a zero header means "no state": the inverse is then built from prev_support).  The call
 *          reads it and overwrites it with the state of the support it returns.  It is built again
 *          from nothing when prev_support is not the set the state was left for, and every 64 calls
 *          (rounding errors of the corrections add up from token to token).
 * Other arguments, failure of a row (its state is then cleared) and supported shapes as for
 * cs_recover_support_inc.
 */
size_t cs_inc_state_words(int k);
cs_status cs_recover_support_inc_carry(cs_ctx* ctx, const cs_op* op, const cs_dict* dict, int k,
                                       const float* y, int B,
                                       const int32_t* prev_support, int swaps, uint32_t* state,
                                       int32_t* support, float* coef, float* resid_norm, float* margin);

/*
 * Block-sparse gated (SwiGLU) feed-forward layer restricted to the support
 * (masked execution of Sec. 3; block sparsity of Sec. 7):
 *   out[t] = sum_{g in S_t} Wd_g ( silu(Wg_g x_t) * (Wu_g x_t) ),  silu(u) = u/(1+exp(-u)).
 *   Wg, Wu: [G][b][d]  (unit g, channel c: one contiguous row of d inputs)
 *   Wd:     [G][d][b]  (unit g, output row j: the b channel weights, contiguous)
 *   x:      [T][d] in, out: [T][d] out, both of type `dtype` (float or bf16 bits)
 *   support: int32[k] if shared != 0 (one support for all T rows: task-conditioned
 *            prefill, Sec. 4), else int32[T][k] (token-adaptive decode, Sec. 5);
 *            entries distinct within a row and in [0, G).  Order is irrelevant.
 * Accumulation is in fp32.  On the bf16 paths the hidden values silu(Wg x) * (Wu x) are stored as bf16
 * between the two products (the second accumulation sees bf16 inputs) and the result is rounded to bf16 once.
 * Requires d % 8 == 0 and b % 8 == 0.  An out-of-range support entry makes that
 * unit contribute nothing (it is never dereferenced).
 */
cs_status cs_block_ffn(cs_ctx* ctx, int dtype, const void* Wg, const void* Wu, const void* Wd,
                       int d, int G, int b, const void* x, int T,
                       const int32_t* support, int k, int shared, void* out);

/*
 * cs_block_ffn for callers that cannot allocate device memory and must not depend on a buffer that was
 * allocated for them: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same kernels and same results as cs_block_ffn; the only difference is the workspace
 * for the values handed from the first product to the second, which is a fixed array of
 * CS_STATIC_SCRATCH_BYTES bytes in the library's device image instead of the context's scratch buffer.
 * Every GPU the library runs on holds one copy of that array until the process ends.  The call itself
 * allocates and frees nothing.  Shapes whose workspace exceeds the array return CS_ENOMEM with a message
 * (the decode shapes fit: T <= 16 rows of bf16, up to 1024 units of 64 channels; long prefill batches
 * do not).  All calls on one GPU share the array, whatever their context or stream: two such calls that
 * overlap in time on one GPU race.  Nothing in it has to be zero at entry; each call overwrites what
 * it reads.
 */
#define CS_STATIC_SCRATCH_BYTES (4u << 20)
cs_status cs_block_ffn_static(cs_ctx* ctx, int dtype, const void* Wg, const void* Wu, const void* Wd,
                              int d, int G, int b, const void* x, int T,
                              const int32_t* support, int k, int shared, void* out);

/*
 * Head-pruned single-query (decode) attention over a key/value cache: heads are
 * the structured units (Sec. 3, Sec. 7).  For every kept head h of sequence i:
 *   out[i][h] = softmax(q[i][h] . K[i][h][:]^T / sqrt(dh)) V[i][h][:]
 * over all L cached positions (no mask, no positional transform); pruned heads
 * output zeros.
 *   q: [B][H][dh], K, V: [B][H][L][dh], out: [B][H][dh], all of type `dtype`
 *   heads: int32[B][kh], distinct, in [0, H).
 * Requires dh in {64, 128, 256}, L >= 1.
 */
cs_status cs_head_attn(cs_ctx* ctx, int dtype, const void* q, const void* K, const void* V,
                       int B, int H, int L, int dh, const int32_t* heads, int kh, void* out);

/*
 * Joint prompt-token and unit selection (Sec. 6): from a sketch of per-token
 * saliency and a sketch of channel usage, return the retained tokens and the
 * channel support in one call.
 *   tokens  = indices of the k_tok largest entries of the back-projection
 *             p = Phi_tok^T y_tok (signed; ties -> smaller index), ascending;
 *   support = cs_recover_support(ch_op, ch_dict, k_ch) applied to y_ch.
 *   y_tok: float[tok_op->m], y_ch: float[ch_op->m]
 *   tokens: int32[k_tok] out, support: int32[k_ch] out
 *   resid_norm, margin: float[1] out or NULL (of the channel recovery)
 * Requires 1 <= k_tok <= tok_op->n.
 */
cs_status cs_joint_select(cs_ctx* ctx, const cs_op* tok_op, const float* y_tok, int k_tok,
                          const cs_op* ch_op, const cs_dict* ch_dict, const float* y_ch, int k_ch,
                          int32_t* tokens, int32_t* support, float* resid_norm, float* margin);

/*
 * Coupled joint selection (Sec. 6: removing a token changes the latent measurements and
 * therefore the recovered support; constraint z_t = A_t(r) Psi(r) alpha_t).  The smallest
 * procedure with that coupling:
 *   tokens  = as cs_joint_select;
 *   ybar    = mean over the retained tokens t of Y_ch[t][:] (by linearity of the sketch,
 *             the sketch of the retained tokens' mean usage);
 *   support = cs_recover_support(ch_op, ch_dict, k_ch) applied to ybar.
 *   y_tok:  float[tok_op->m]
 *   Y_ch:   float[tok_op->n][ch_op->m], one channel sketch per prompt token
 *   tokens: int32[k_tok] out, support: int32[k_ch] out
 *   ybar:   float[ch_op->m] out or NULL
 *   resid_norm, margin: float[1] out or NULL (of the channel recovery)
 * The rows are summed in a fixed order (chunks of 64 retained tokens, then the chunks), so
 * the result does not depend on timing.
 */
cs_status cs_joint_select_coupled(cs_ctx* ctx, const cs_op* tok_op, const float* y_tok, int k_tok,
                                  const cs_op* ch_op, const cs_dict* ch_dict, const float* Y_ch, int k_ch,
                                  int32_t* tokens, int32_t* support, float* ybar,
                                  float* resid_norm, float* margin);

/*
 * Uncertainty-driven measurement budget (Sec. 8.1).  cs_softmax_entropy returns, for every
 * row of logits, the entropy in nats of the predictive distribution p = softmax(logits),
 *   H(p) = - sum_v p(v) ln p(v);
 * cs_uds_budget is the controller itself (host arithmetic, no device work),
 *   m_t = clip( floor( m_base (1 + gamma H) ), m_min, m_max ),
 * whose result is the `m` of the next step's cs_op (rows of Phi are nested in m).
 *   logits: device float[B][V], entropy: device float[B] out; V >= 1.
 * cs_uds_budget returns the budget, or -1 if m_min > m_max, m_min < 1 or an argument is not finite.
 */
cs_status cs_softmax_entropy(cs_ctx* ctx, const float* logits, int B, int V, float* entropy);
int32_t cs_uds_budget(int32_t m_base, float gamma, float entropy, int32_t m_min, int32_t m_max);

/*
 * Diagnostic, not a step of the method: read `bytes` bytes of device memory once, 16 bytes per lane, and
 * xor every 32-bit word read into checksum[0] (atomically; zero it beforehand to get the xor of the
 * buffer; a trailing bytes % 16 is not read).  The duration of this call is what a plain streaming read
 * reaches on the device.  Sec. 14 and Sec. 15 ask for latency on real hardware, where the
 * bandwidth-bound calls (decode FFN, attention over the cache) are limited by the memory system; the
 * benchmark reports their bandwidth against the published peak and against this measured ceiling.
 *   src: device pointer, 16-byte aligned;  checksum: device uint32_t[1].
 */
cs_status cs_stream_read(cs_ctx* ctx, const void* src, size_t bytes, uint32_t* checksum);

/*
 * Token-selection operator of Sec. 6 (the retained prompt x~ = Pi(r) x): copy the rows
 * of x named by `tokens` into a dense matrix, in the order given.
 *   x: [n_rows][d] in, tokens: int32[k_tok] with entries in [0, n_rows), out: [k_tok][d] out,
 *   both of type `dtype`.  Requires d % 8 == 0.  An out-of-range entry yields a zero row.
 */
cs_status cs_gather_rows(cs_ctx* ctx, int dtype, const void* x, int n_rows, int d,
                         const int32_t* tokens, int k_tok, void* out);

#ifdef __cplusplus
}
#endif
#endif /* CS_H_ */
