// Token side of the joint selection (paper Sec. 6): back-projection of the token
// sketch, p = Phi^T y, and selection of the k largest entries (ties -> smaller
// index) returned in ascending index order.
#include "kernels.hpp"
#include "common.hpp"

namespace csk {

// Hadamard ensemble: one thread per column; Gaussian ensemble: one thread per group of four columns
// (one Philox call); rows are visited in ascending order.
__global__ void backproject_kernel(OpDesc op, const float* __restrict__ y, float* __restrict__ p) {
    extern __shared__ float ys[];
    for (int i = threadIdx.x; i < op.m; i += blockDim.x) ys[i] = y[i];
    __syncthreads();
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (op.ens == 2) {                                   // Hadamard ensemble: one thread per column
        if (t >= op.n) return;
        const SrhtRows key = srht_rows_key(op);
        const u32x4 b = srht_sign_bits(op, (uint32_t)t >> 7);
        const uint32_t d = (b.w[((uint32_t)t & 127u) >> 5] >> ((uint32_t)t & 31u)) & 1u;
        float acc = 0.f;
        for (int i = 0; i < op.m; ++i) {
            const uint32_t sgn = ((__popc(srht_row(key, (uint32_t)i) & (uint32_t)t) ^ d) & 1u) << 31;
            acc += __uint_as_float(__float_as_uint(ys[i]) ^ sgn);
        }
        p[t] = acc * op.scale;
    } else {
        const int c0 = t * 4;
        if (c0 >= op.n) return;
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int i = 0; i < op.m; ++i) {
            float e[4];
            gauss4(op, (uint32_t)i, (uint32_t)t, e);
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] += e[j] * ys[i];
        }
        for (int j = 0; j < 4 && c0 + j < op.n; ++j) p[c0 + j] = acc[j] * op.scale;
    }
}

// Rademacher ensemble: one Philox call gives the signs of 128 columns of a row, so a workgroup owns a
// group of 128 columns and draws every (row, group) word once into LDS; thread (q, c) then sums the
// rows of quarter q of each row block for column c in ascending order, and the four quarter sums are
// added in a fixed order.
constexpr int BP_THREADS = 512;
constexpr int BP_ROWS = 1024;                 // rows per block: 16 KB of sign words + 4 KB of y
__global__ __launch_bounds__(BP_THREADS)
void backproject_rademacher_kernel(OpDesc op, const float* __restrict__ y, float* __restrict__ p) {
    __shared__ uint32_t bits[BP_ROWS][4];
    __shared__ float ys[BP_ROWS];
    __shared__ float quarter[4][128];
    const int tid = threadIdx.x, c = tid & 127, q = tid >> 7;
    const uint32_t cg = blockIdx.x;
    const int word = c >> 5, bit = c & 31;
    float acc = 0.f;
    for (int r0 = 0; r0 < op.m; r0 += BP_ROWS) {
        const int nr = min(BP_ROWS, op.m - r0);
        for (int i = tid; i < nr; i += BP_THREADS) {
            const u32x4 b = rademacher_bits(op, (uint32_t)(r0 + i), cg);
            bits[i][0] = b.w[0]; bits[i][1] = b.w[1]; bits[i][2] = b.w[2]; bits[i][3] = b.w[3];
            ys[i] = y[r0 + i];
        }
        __syncthreads();
        const int per = (nr + 3) >> 2;
        const int i1 = min(nr, (q + 1) * per);
        for (int i = q * per; i < i1; ++i) {
            const uint32_t sgn = ((bits[i][word] >> bit) & 1u) << 31;
            acc += __uint_as_float(__float_as_uint(ys[i]) ^ sgn);
        }
        __syncthreads();
    }
    quarter[q][c] = acc;
    __syncthreads();
    const int col = (int)cg * 128 + c;
    if (q == 0 && col < op.n) p[col] = (((quarter[0][c] + quarter[1][c]) + quarter[2][c]) + quarter[3][c]) * op.scale;
}

hipError_t launch_backproject(const OpDesc& op, const float* y, float* p, hipStream_t s) {
    if (op.ens == 1) {
        hipLaunchKernelGGL(backproject_rademacher_kernel, dim3((op.n + 127) / 128), dim3(BP_THREADS), 0, s, op, y, p);
        return hipGetLastError();
    }
    const int items = op.ens != 0 ? op.n : (op.n + 3) / 4;
    const int block = 64;                    // many small workgroups: the row loop is long
    hipLaunchKernelGGL(backproject_kernel, dim3((items + block - 1) / block), dim3(block),
                       (size_t)op.m * sizeof(float), s, op, y, p);
    return hipGetLastError();
}

// order-preserving map float -> uint32 (larger float <=> larger key)
__device__ __forceinline__ uint32_t float_key(float f) {
    uint32_t u = __float_as_uint(f);
    if (u == 0x80000000u) u = 0u;            // -0 and +0 compare equal
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int TK_THREADS = 1024;

// Radix select of the k-th largest key (four 8-bit passes), then an order-keeping
// compaction: everything above the threshold, plus the first `need` entries equal
// to it.  One workgroup; the scores are re-read from L2 in every pass.
__global__ __launch_bounds__(TK_THREADS)
void topk_kernel(const float* __restrict__ scores, int n, int k, int32_t* __restrict__ out) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sh_prefix, sh_need;
    __shared__ uint32_t wtot[4];
    __shared__ uint32_t wsum_gt[TK_THREADS / 64], wsum_eq[TK_THREADS / 64];
    __shared__ uint32_t base_gt, base_eq;
    const int tid = threadIdx.x;

    uint32_t prefix = 0, mask = 0, need = (uint32_t)k;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < n; i += TK_THREADS) {
            const uint32_t key = float_key(scores[i]);
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        // the bin that holds the need-th largest of the candidates: bins are scanned from the top by a
        // suffix sum over the 256 counts (4 waves), exactly one bin has "at least need at or above it,
        // fewer than need above it"
        uint32_t h = 0, sfx = 0;
        if (tid < 256) {
            h = hist[tid];
            sfx = h;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t o = __shfl_down(sfx, off, 64);
                if ((tid & 63) + off < 64) sfx += o;
            }
            if ((tid & 63) == 0) wtot[tid >> 6] = sfx;
        }
        __syncthreads();
        if (tid < 256) {
            uint32_t above = 0;
            for (int w = (tid >> 6) + 1; w < 4; ++w) above += wtot[w];
            const uint32_t at_or_above = sfx + above, strictly_above = at_or_above - h;
            if (at_or_above >= need && strictly_above < need) {
                sh_prefix = prefix | ((uint32_t)tid << shift);
                sh_need = need - strictly_above;      // how many are still wanted inside this bin
            }
        }
        __syncthreads();
        prefix = sh_prefix;
        need = sh_need;
        mask |= 255u << shift;
        __syncthreads();
    }
    const uint32_t thr = prefix;            // key of the k-th largest; `need` equal keys are kept

    if (tid == 0) { base_gt = 0; base_eq = 0; }
    __syncthreads();
    const int lane = tid & 63, wave = tid >> 6;
    for (int i0 = 0; i0 < n; i0 += TK_THREADS) {
        const int i = i0 + tid;
        uint32_t key = 0;
        bool gt = false, eq = false;
        if (i < n) { key = float_key(scores[i]); gt = key > thr; eq = key == thr; }
        const unsigned long long bgt = __ballot(gt), beq = __ballot(eq);
        const unsigned long long below = (1ull << lane) - 1ull;
        const uint32_t lgt = __popcll(bgt & below), leq = __popcll(beq & below);
        if (lane == 0) { wsum_gt[wave] = __popcll(bgt); wsum_eq[wave] = __popcll(beq); }
        __syncthreads();
        uint32_t ogt = base_gt, oeq = base_eq;
        for (int w = 0; w < wave; ++w) { ogt += wsum_gt[w]; oeq += wsum_eq[w]; }
        const uint32_t gt_before = ogt + lgt, eq_before = oeq + leq;
        if (gt) out[gt_before + min(eq_before, need)] = i;
        else if (eq && eq_before < need) out[gt_before + eq_before] = i;
        __syncthreads();
        if (tid == 0) {
            uint32_t a = 0, b = 0;
            for (int w = 0; w < TK_THREADS / 64; ++w) { a += wsum_gt[w]; b += wsum_eq[w]; }
            base_gt += a; base_eq += b;
        }
        __syncthreads();
    }
}

// Token-selection operator: gather the kept rows.  One workgroup per output row.
__global__ void gather_rows_kernel(const uint4* __restrict__ x, int n_rows, int chunks, const int32_t* __restrict__ tokens,
                                   uint4* __restrict__ out) {
    const int r = blockIdx.x;
    const int src = tokens[r];
    const bool ok = src >= 0 && src < n_rows;
    for (int c = threadIdx.x; c < chunks; c += blockDim.x)
        out[(size_t)r * chunks + c] = ok ? x[(size_t)src * chunks + c] : make_uint4(0u, 0u, 0u, 0u);
}

hipError_t launch_gather_rows(const void* x, int n_rows, size_t row_bytes, const int32_t* tokens, int k_tok,
                              void* out, hipStream_t s) {
    if (k_tok <= 0) return hipSuccess;
    hipLaunchKernelGGL(gather_rows_kernel, dim3(k_tok), dim3(256), 0, s, reinterpret_cast<const uint4*>(x), n_rows,
                       (int)(row_bytes / 16), tokens, reinterpret_cast<uint4*>(out));
    return hipGetLastError();
}

// Mean of the listed rows of Y [n_rows][m] in a fixed order: a workgroup sums a chunk of 64 listed
// rows (thread = column), a second kernel adds the chunk sums in order and scales.
constexpr int PL_CHUNK = 64;
__global__ __launch_bounds__(256)
void pool_rows_partial_kernel(const float* __restrict__ Y, int n_rows, int m, const int32_t* __restrict__ tokens,
                              int k_tok, float* __restrict__ partial) {
    const int c = blockIdx.y * 256 + threadIdx.x;
    if (c >= m) return;
    const int i0 = blockIdx.x * PL_CHUNK, i1 = min(k_tok, i0 + PL_CHUNK);
    float acc = 0.f;
    for (int i = i0; i < i1; ++i) {
        const int t = tokens[i];
        if (t >= 0 && t < n_rows) acc += Y[(size_t)t * m + c];
    }
    partial[(size_t)blockIdx.x * m + c] = acc;
}
__global__ __launch_bounds__(256)
void pool_rows_final_kernel(const float* __restrict__ partial, int nchunks, int m, float scale, float* __restrict__ ybar,
                            float* __restrict__ copy) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= m) return;
    float acc = 0.f;
    for (int q = 0; q < nchunks; ++q) acc += partial[(size_t)q * m + c];
    ybar[c] = acc * scale;
    if (copy) copy[c] = acc * scale;
}

size_t pool_rows_scratch_floats(int m, int k_tok) { return (size_t)((k_tok + PL_CHUNK - 1) / PL_CHUNK) * m; }

hipError_t launch_pool_rows(const float* Y, int n_rows, int m, const int32_t* tokens, int k_tok, float* partial,
                            float* ybar, float* copy, hipStream_t s) {
    const int nchunks = (k_tok + PL_CHUNK - 1) / PL_CHUNK, cb = (m + 255) / 256;
    hipLaunchKernelGGL(pool_rows_partial_kernel, dim3(nchunks, cb), dim3(256), 0, s, Y, n_rows, m, tokens, k_tok, partial);
    hipLaunchKernelGGL(pool_rows_final_kernel, dim3(cb), dim3(256), 0, s, partial, nchunks, m, 1.0f / (float)k_tok, ybar, copy);
    return hipGetLastError();
}

// Entropy of softmax(logits) per row (paper Sec. 8.1).  With mx a reference value, S = sum exp(x - mx)
// and T = sum (x - mx) exp(x - mx), the entropy is ln S - T / S.  A row is cut into slices so that a few
// rows still fill the chip: one workgroup reduces a slice to (mx, S, T) with mx the slice maximum, and a
// second kernel merges the slices of a row in a fixed order: moving the reference from m1 to M scales
// S1 by e^(m1-M) and turns T1 into (T1 + (m1 - M) S1) e^(m1-M).
constexpr int EN_THREADS = 256;
constexpr int EN_SLICE = 8192;                          // logits per workgroup
__global__ __launch_bounds__(EN_THREADS)
void softmax_entropy_slice_kernel(const float* __restrict__ logits, int V, int nslices, float* __restrict__ part) {
    __shared__ float red[2][EN_THREADS / 64];
    const int row = blockIdx.y, sl = blockIdx.x;
    const float* x = logits + (size_t)row * V;
    const int i0 = sl * EN_SLICE, i1 = min(V, i0 + EN_SLICE);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // the slice is read once: 32 logits per thread, all loads in flight before the first use
    constexpr int PER = EN_SLICE / EN_THREADS;
    float v[PER];
    if ((V & 3) == 0) {                                 // 16-byte aligned rows
#pragma unroll
        for (int q = 0; q < PER / 4; ++q) {
            const int i = i0 + (q * EN_THREADS + tid) * 4;
            float4 t = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            if (i < i1) t = *reinterpret_cast<const float4*>(x + i);      // i1 - i is a multiple of 4 here
            v[4 * q] = t.x; v[4 * q + 1] = t.y; v[4 * q + 2] = t.z; v[4 * q + 3] = t.w;
        }
    } else {
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int i = i0 + q * EN_THREADS + tid;
            v[q] = i < i1 ? x[i] : -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int q = 0; q < PER; ++q) mx = fmaxf(mx, v[q]);
    mx = wave_max(mx);
    if (lane == 0) red[0][wave] = mx;
    __syncthreads();
    mx = red[0][0];
    for (int w = 1; w < EN_THREADS / 64; ++w) mx = fmaxf(mx, red[0][w]);
    __syncthreads();
    float S = 0.f, T = 0.f;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const float d = v[q] - mx;                      // padding: -inf, contributes nothing
        const float e = __expf(d);
        S += e;
        if (e > 0.f) T += d * e;                       // exp underflow: the term is 0, not (-inf) * 0
    }
    S = wave_sum(S);
    T = wave_sum(T);
    if (lane == 0) { red[0][wave] = S; red[1][wave] = T; }
    __syncthreads();
    if (tid == 0) {
        float s = 0.f, t = 0.f;
        for (int w = 0; w < EN_THREADS / 64; ++w) { s += red[0][w]; t += red[1][w]; }
        float* o = part + ((size_t)row * nslices + sl) * 3;
        o[0] = mx; o[1] = s; o[2] = t;
    }
}
__global__ void softmax_entropy_merge_kernel(const float* __restrict__ part, int B, int nslices, float* __restrict__ entropy) {
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= B) return;
    const float* p = part + (size_t)row * nslices * 3;
    float M = p[0];
    for (int q = 1; q < nslices; ++q) M = fmaxf(M, p[3 * q]);
    float S = 0.f, T = 0.f;
    for (int q = 0; q < nslices; ++q) {
        const float dm = p[3 * q] - M;                 // <= 0; -inf - (-inf) cannot occur: logits are finite
        const float sc = __expf(dm);
        if (sc > 0.f) {
            S += p[3 * q + 1] * sc;
            T += (p[3 * q + 2] + dm * p[3 * q + 1]) * sc;
        }
    }
    entropy[row] = logf(S) - T / S;
}

size_t softmax_entropy_scratch_floats(int B, int V) { return (size_t)B * ((V + EN_SLICE - 1) / EN_SLICE) * 3; }

hipError_t launch_softmax_entropy(const float* logits, int B, int V, float* part, float* entropy, hipStream_t s) {
    if (B <= 0) return hipSuccess;
    const int nslices = (V + EN_SLICE - 1) / EN_SLICE;
    hipLaunchKernelGGL(softmax_entropy_slice_kernel, dim3(nslices, B), dim3(EN_THREADS), 0, s, logits, V, nslices, part);
    hipLaunchKernelGGL(softmax_entropy_merge_kernel, dim3((B + 63) / 64), dim3(64), 0, s, part, B, nslices, entropy);
    return hipGetLastError();
}

hipError_t launch_topk(const float* scores, int n, int k, int32_t* out, hipStream_t s) {
    hipLaunchKernelGGL(topk_kernel, dim3(1), dim3(TK_THREADS), 0, s, scores, n, k, out);
    return hipGetLastError();
}

}  // namespace csk
