// Host-callable launchers of the HIP kernels (internal to the library).  Host-side declarations only:
// the C ABI (cs_api.hip) needs nothing else, which also lets its argument checking and bookkeeping be
// built for the host alone, against stand-in launchers, and run under the address and
// undefined-behaviour sanitizers on a machine without a GPU.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "op_desc.hpp"

namespace csk {

// y[B][m] = Phi z[B][n]
hipError_t launch_sketch(const OpDesc& op, const float* z, int B, float* y, hipStream_t s);
// scratch: optional workspace (device) for launches that split the columns over several workgroups per tile
hipError_t launch_sketch_multi(const OpDesc* ops, int n_ops, const float* z, int B, float* y, hipStream_t s,
                               void* scratch = nullptr, size_t scratch_bytes = 0);
// the fast transform of the Hadamard ensemble keeps the padded vector in LDS
bool sketch_srht_supported(const OpDesc& op);

// Plan of an (operator, dictionary) pair, all device memory owned by the context.
struct Plan {
    OpDesc op;
    int G, b, rb;
    int N;                // number of atoms = G*rb
    int weighted;         // 1: per-unit triangular weights (dictionary given), 0: raw energy
    float* Mt;            // [N][m]  atoms, contiguous per atom
    float* Mr;            // [m][N]  the same matrix, contiguous per measurement row
    float* gram;          // [N][N]
    float* W;             // [G][rb][rb] lower-triangular score weights (weighted only)
};
hipError_t launch_plan_build(const Plan& p, const float* psi, hipStream_t s);

struct RecoverArgs {
    const float* y; int B; int k;
    int32_t* support; float* coef; float* resid; float* margin;
    float* spill;         // global workspace for the running factor if it does not fit in LDS
    size_t spill_stride;  // floats per problem
    // Several operators in one launch: plans[j] (device array of nplans plans of identical shape) serves
    // problems j*B .. j*B+B-1 of y and of the outputs.  nullptr: the plan passed by value serves all B.
    const Plan* plans = nullptr;
    int nplans = 1;
};
// bytes of global spill workspace needed per problem (0 if everything fits in LDS)
size_t recover_spill_floats(const Plan& p, int k, int lds_limit);
hipError_t launch_recover(const Plan& p, const RecoverArgs& a, int lds_limit, hipStream_t s);

// block iterative hard thresholding (iht.hip): one atom per unit, k <= 64, N <= 512
bool recover_iht_supported(const Plan& p, int k, int lds_limit);
hipError_t launch_recover_iht(const Plan& p, const RecoverArgs& a, int iters, int lds_limit, hipStream_t s);

// warm-started recovery around the previous support (inc.hip): one atom per unit, k <= 64, N <= 512
struct IncArgs {
    const int32_t* prev_support;   // [B][k]
    const float* prev_coef;        // [B][k] in the order of prev_support, or nullptr
    float gamma;                   // weight of the pull towards prev_coef in the first refit
    int swaps;                     // units that may leave and enter
    uint32_t* state = nullptr;     // carried state, [B][state_stride] words (launch_recover_carry only)
    size_t state_stride = 0;
};
// 32-bit words of carried state per sketch: header, age, the list of k units, the k x k inverse of their Gram matrix
size_t recover_inc_state_words(int k);
hipError_t launch_recover_carry(const Plan& p, const RecoverArgs& a, const IncArgs& q, int lds_limit, hipStream_t s);
bool recover_inc_supported(const Plan& p, int k, int lds_limit);
hipError_t launch_recover_inc(const Plan& p, const RecoverArgs& a, const IncArgs& q, int lds_limit, hipStream_t s);

// p[n] = Phi^T y (back-projection), then top-k.
hipError_t launch_backproject(const OpDesc& op, const float* y, float* p, hipStream_t s);
hipError_t launch_topk(const float* scores, int n, int k, int32_t* out, hipStream_t s);

// ybar[m] (and `copy`, if not null) = mean over the listed rows of Y [n_rows][m];
// partial: pool_rows_scratch_floats(m, k_tok) floats
size_t pool_rows_scratch_floats(int m, int k_tok);
hipError_t launch_pool_rows(const float* Y, int n_rows, int m, const int32_t* tokens, int k_tok, float* partial,
                            float* ybar, float* copy, hipStream_t s);

// entropy[B] = entropy in nats of softmax(logits[B][V]) per row; part: softmax_entropy_scratch_floats floats
size_t softmax_entropy_scratch_floats(int B, int V);
hipError_t launch_softmax_entropy(const float* logits, int B, int V, float* part, float* entropy, hipStream_t s);

// out[i][:] = x[tokens[i]][:], rows of `row_bytes` bytes (a multiple of 16)
hipError_t launch_gather_rows(const void* x, int n_rows, size_t row_bytes, const int32_t* tokens, int k_tok,
                              void* out, hipStream_t s);
// zero `bytes` bytes (a multiple of 4) with a kernel, so that the call can be captured in a graph
hipError_t launch_zero_fill(void* dst, size_t bytes, hipStream_t s);

// xor of all 32-bit words of the first bytes/16*16 bytes of src into *checksum (atomically; the caller zeroes it)
hipError_t launch_stream_read(const void* src, size_t bytes, uint32_t* checksum, hipStream_t s);

struct FfnArgs {
    int dtype;            // 0 f32, 1 bf16
    const void *Wg, *Wu, *Wd; int d, G, b;
    const void* x; int T; const int32_t* support; int k; int shared;
    void* out;
    void* scratch; size_t scratch_bytes;
    int union_hint = 0;   // 0: guess from T, k, G whether the rows' supports cover all units; 1: they do; 2: they do not
};
size_t ffn_scratch_bytes(const FfnArgs& a);
// many-row path on the matrix cores (ffn_gemm.hip)
bool ffn_gemm_ok(const FfnArgs& a);
size_t ffn_gemm_scratch_bytes(const FfnArgs& a);
hipError_t launch_ffn_gemm(const FfnArgs& a, hipStream_t s);
// token-adaptive batches of 17 to 64 rows (ffn_wide.hip)
bool ffn_wide_ok(const FfnArgs& a);
size_t ffn_wide_scratch_bytes(const FfnArgs& a);
hipError_t launch_ffn_wide(const FfnArgs& a, hipStream_t s);
hipError_t launch_block_ffn(const FfnArgs& a, hipStream_t s);

struct AttnArgs {
    int dtype;
    const void *q, *K, *V; int B, H, L, dh;
    const int32_t* heads; int kh; void* out;
    void* scratch; size_t scratch_bytes;
};
size_t attn_scratch_bytes(const AttnArgs& a);
hipError_t launch_head_attn(const AttnArgs& a, hipStream_t s);

}  // namespace csk
