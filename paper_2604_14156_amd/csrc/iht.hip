// Structured sparse recovery by block iterative hard thresholding (paper Sec. 8:
// proximal steps followed by a projection, a small fixed number of iterations; projection
// onto exactly k units, Sec. 7).  One workgroup per sketch, one atom per unit.
//
// Everything runs in the Gram domain (G = M^T M in LDS, c0 = M^T y): the gradient is
// g = c0 - G alpha, the exact line-search step on the current support is
// mu = ||g_S||^2 / (g_S^T G g_S), and the projection keeps the k units with the largest
// weighted energy (w_c p_c)^2.  The k largest are found by rank counting: every atom
// counts how many atoms beat it (ties -> smaller index); the count is split over the
// idle threads of the workgroup and summed with integer LDS atomics, so the result
// does not depend on timing.  After the last iteration the coefficients are refitted
// by least squares on the final support (Cholesky factor of G_SS built in LDS by one
// wavefront, then one refinement step against the explicit residual).
#include "kernels.hpp"
#include "common.hpp"
#include "small_dense.hpp"
#include "gram_loads.hpp"

namespace csk {

constexpr int IH_MAXK = 64;
constexpr int IH_THREADS = 512;

struct IhtLayout {
    int off_y, off_r, off_alpha, off_g, off_e, off_cnt, off_S, off_t, off_L, off_misc, off_gram, off_stage;
    int total_floats;
};

static bool make_iht_layout(const Plan& p, int k, int lds_limit, int nthreads, IhtLayout& L) {
    const int N = p.N, m = p.op.m;
    const int Np = (N + 7) & ~7;
    int o = 0;
    L.off_y = o; o += (m + 3) & ~3;
    L.off_r = o; o += (m + 3) & ~3;
    L.off_alpha = o; o += Np;
    L.off_g = o; o += Np;
    L.off_e = o; o += Np;
    L.off_cnt = o; o += Np;
    L.off_S = o; o += IH_MAXK;
    L.off_t = o; o += 4 * IH_MAXK;
    L.off_L = o; o += IH_MAXK * (IH_MAXK + 1);
    L.off_misc = o; o += 32;
    L.off_stage = o; o += nthreads * 4;
    L.off_gram = -1;
    const long limit = lds_limit / 4 - 16;
    if (o > limit) return false;
    if ((long)o + (long)N * N <= limit) { L.off_gram = o; o += N * N; }
    L.total_floats = o;
    return true;
}

template <bool GRAM_LDS>
__global__ __launch_bounds__(IH_THREADS)
void recover_iht_kernel(Plan p, RecoverArgs a, int iters, IhtLayout L) {
    extern __shared__ float lds[];
    const int tid = threadIdx.x, NT = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nwaves = NT >> 6;
    const int prob = blockIdx.x;
    const int N = p.N, m = p.op.m, k = a.k;
    const bool active = tid < N;

    float* yv = lds + L.off_y;
    float* rv = lds + L.off_r;
    float* alpha = lds + L.off_alpha;
    float* gl_ = lds + L.off_g;
    float* en = lds + L.off_e;
    int* cnt = reinterpret_cast<int*>(lds + L.off_cnt);
    int* S = reinterpret_cast<int*>(lds + L.off_S);
    float* tv = lds + L.off_t;                  // [4][IH_MAXK] small vectors of the refit
    float* Lf = lds + L.off_L;                  // Cholesky factor, row stride IH_MAXK + 1
    float* misc = lds + L.off_misc;
    float* stage = lds + L.off_stage;
    float* gram_l = lds + L.off_gram;
    const float* gram = GRAM_LDS ? gram_l : p.gram;

    // ---- loads: sketch, weight, Gram matrix, c0 = M^T y
    const float* y = a.y + (size_t)prob * m;
    int bad = 0;
    float w = 1.f;                                     // atom norm: W holds 1/norm
    if (active && p.weighted) { const float iw = p.W[tid]; w = iw > 0.f ? 1.0f / iw : 0.f; }
    const float c0 = load_sketch_gram_c0<GRAM_LDS>(p, y, yv, gram_l, stage, bad);
    if (active) alpha[tid] = 0.f;
    // helpers of the rank count: thread (c, part) scans a slice of the candidates
    const int Npad = (N + 63) & ~63;
    const int rparts = NT / Npad > 0 ? NT / Npad : 1;
    const int rc = tid % Npad, rpart = tid / Npad;
    const int Np8 = (N + 7) & ~7;
    const int rper = (((N + rparts - 1) / rparts) + 7) & ~7;
    for (int i = N + tid; i < Np8; i += NT) en[i] = -1.f;   // padding never beats anything (energies are >= 0)
    __syncthreads();

    float margin = 1.f;
    // rank all atoms by the energies in en[]; returns this thread's rank (threads with tid < N)
    auto rank_atoms = [&]() -> int {
        if (tid < N) cnt[tid] = 0;
        __syncthreads();
        if (rpart < rparts && rc < N) {
            const float mine = en[rc];
            const int j0 = rpart * rper, j1 = min(Np8, j0 + rper);     // rper is a multiple of 8
            int beat = 0;
            for (int j = j0; j < j1; j += 8) {
                const float4 a0 = *reinterpret_cast<const float4*>(en + j);
                const float4 a1 = *reinterpret_cast<const float4*>(en + j + 4);
                const float o[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
                for (int q = 0; q < 8; ++q) beat += (int)(o[q] > mine) | ((int)(o[q] == mine) & (int)(j + q < rc));   // no branches
            }
            if (beat) atomicAdd(&cnt[rc], beat);
        }
        __syncthreads();
        return active ? cnt[tid] : 0x7fffffff;
    };

    float pmine = 0.f;
    float num0 = 0.f;                               // ||g_S||^2 of the first iteration (wave 0)
    for (int it = 0; it < iters; ++it) {
        // gradient g = c0 - G alpha (alpha has at most k non-zeros, listed in S after the first pass).
        // Each wave keeps the list and the listed coefficients in the registers of its first k lanes and
        // hands them out by scalar lane reads, so the k Gram reads below are independent of each other.
        float g = c0;
        if (it > 0) {
            const int sreg = lane < k ? S[lane] : 0;
            const float areg = lane < k ? alpha[sreg] : 0.f;
            float acc = 0.f;
            const int ta = active ? tid : 0;
            for (int j = 0; j < k; j += 4) {
                float gv4[4], av4[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {       // lanes >= k hold index 0 and coefficient 0; j + q <= 63
                    const int sj = __builtin_amdgcn_readlane(sreg, j + q);
                    av4[q] = readlane_f32(areg, j + q);
                    gv4[q] = gram[(size_t)sj * N + ta];
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) acc += av4[q] * gv4[q];
            }
            g -= acc;
        }
        if (active) gl_[tid] = g;
        if (it == 0) {
            float e = w * g; e = e * e;
            if (!(e >= 0.f)) e = 0.f;
            if (active) en[tid] = e;
            __syncthreads();
            const int r0 = rank_atoms();
            if (r0 < k) S[r0] = tid;
        }
        __syncthreads();
        // step length on the current support: one wavefront, lane j owns S[j]
        if (wave == 0) {
            const int sreg = lane < k ? S[lane] : 0;
            const float greg = lane < k ? gl_[sreg] : 0.f;
            float t = 0.f;
            for (int i = 0; i < k; i += 4) {
                float gv4[4], gi4[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int si = __builtin_amdgcn_readlane(sreg, i + q);
                    gi4[q] = readlane_f32(greg, i + q);
                    gv4[q] = gram[(size_t)si * N + sreg];
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) t += gv4[q] * gi4[q];
            }
            const float num = wave_sum(greg * greg), den = wave_sum(greg * t);
            if (it == 0) num0 = num;
            // Once the gradient on the support has dropped to 1e-3 of its first value, alpha is the least-squares fit
            // on that support to three digits (the refit after the loop makes it exact) and further steps only
            // shrink a vector whose direction fp32 resolves less and less: the step length, and with it the
            // energies of the units outside the support and the margin, would come to depend on rounding.  The
            // iteration stops there (support, alpha and margin stand).
            const bool converged = it > 0 && num <= 1e-6f * num0;
            if (lane == 0) { misc[0] = den > 0.f ? num / den : 0.f; misc[3] = converged ? 1.f : 0.f; }
        }
        __syncthreads();
        if (misc[3] != 0.f) break;                      // uniform: every thread reads the same word
        const float mu = misc[0];
        pmine = active ? alpha[tid] + mu * g : 0.f;
        float e = w * pmine; e = e * e;
        if (!(e >= 0.f)) e = 0.f;                       // NaN ranks last among equals
        if (active) en[tid] = e;
        __syncthreads();
        const int r = rank_atoms();
        if (active) alpha[tid] = r < k ? pmine : 0.f;
        if (r < k) S[r] = tid;
        if (r == k - 1) misc[1] = e;
        if (r == k) misc[2] = e;
        __syncthreads();
        if (k < p.G) { const float ek = misc[1], ek1 = misc[2]; margin = ek > 0.f ? (ek - ek1) / ek : 0.f; }
        else margin = 1.f;
    }

    const bool want_fit = a.coef != nullptr || a.resid != nullptr;
    float* beta = tv, *xs = tv + IH_MAXK, *gv = tv + 2 * IH_MAXK, *dl = tv + 3 * IH_MAXK;
    if (want_fit) {
        // Cholesky factor of G_SS, one wavefront: lane j builds row j
        if (wave == 0) bad |= wave_cholesky(gram, N, S, k, 0.f, Lf, gv, lane);
        bad = __syncthreads_or(bad);
        auto solve = [&](float rhs) -> float { return wave_cholesky_solve(Lf, k, rhs, lane); };
        if (active) en[tid] = c0;                        // right-hand side c0_S: published through en[]
        __syncthreads();
        if (wave == 0) {
            const float x = solve(lane < k ? en[S[lane]] : 0.f);
            if (lane < k) xs[lane] = x;
        }
        __syncthreads();
        for (int i = tid; i < m; i += NT) {
            float s = yv[i];
            for (int j = 0; j < k; ++j) s -= xs[j] * p.Mr[(size_t)i * N + S[j]];
            rv[i] = s;
        }
        __syncthreads();
        for (int j = wave; j < k; j += nwaves) {
            float s = 0.f;
            for (int i = lane; i < m; i += 64) s += p.Mr[(size_t)i * N + S[j]] * rv[i];
            s = wave_sum(s);
            if (lane == 0) gv[j] = s;
        }
        __syncthreads();
        if (wave == 0) {
            const float d = solve(lane < k ? gv[lane] : 0.f);
            if (lane < k) { xs[lane] += d; dl[lane] = d; }
        }
        __syncthreads();
        float ss = 0.f;
        for (int i = tid; i < m; i += NT) {
            float s = rv[i];
            for (int j = 0; j < k; ++j) s -= dl[j] * p.Mr[(size_t)i * N + S[j]];
            ss += s * s;
        }
        ss = wave_sum(ss);
        if (lane == 0) beta[wave] = ss;                  // beta[] is free: per-wave partial sums
        __syncthreads();
    }
    for (int qi = tid; qi < k; qi += NT) {
        const int gsel = S[qi];
        int rank = 0;
        for (int o = 0; o < k; ++o) rank += S[o] < gsel;
        a.support[(size_t)prob * k + rank] = gsel;
        if (a.coef) a.coef[(size_t)prob * k + rank] = xs[qi];
    }
    if (tid == 0) {
        if (a.resid) {
            float tot = 0.f;
            for (int wv = 0; wv < nwaves; ++wv) tot += beta[wv];
            a.resid[prob] = bad ? __int_as_float(0x7fc00000) : sqrtf(tot);
        }
        if (a.margin) a.margin[prob] = bad ? 0.f : margin;
    }
}

bool recover_iht_supported(const Plan& p, int k, int lds_limit) {
    if (p.rb != 1 || k > IH_MAXK || p.N > IH_THREADS) return false;
    IhtLayout L;
    const int nthreads = (p.N <= 64 && p.op.m <= 64) ? 64 : IH_THREADS;
    return make_iht_layout(p, k, lds_limit, nthreads, L);
}

hipError_t launch_recover_iht(const Plan& p, const RecoverArgs& a, int iters, int lds_limit, hipStream_t s) {
    if (a.B <= 0) return hipSuccess;
    const int nthreads = (p.N <= 64 && p.op.m <= 64) ? 64 : IH_THREADS;
    IhtLayout L;
    if (!make_iht_layout(p, a.k, lds_limit, nthreads, L)) return hipErrorInvalidValue;
    const size_t bytes = (size_t)L.total_floats * 4;
    if (L.off_gram >= 0) {
        static size_t allowed = 0;
        if (bytes > allowed) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(recover_iht_kernel<true>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
            if (e != hipSuccess) return e;
            allowed = bytes;
        }
        hipLaunchKernelGGL(recover_iht_kernel<true>, dim3(a.B), dim3(nthreads), bytes, s, p, a, iters, L);
    } else {
        static size_t allowed = 0;
        if (bytes > allowed) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(recover_iht_kernel<false>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
            if (e != hipSuccess) return e;
            allowed = bytes;
        }
        hipLaunchKernelGGL(recover_iht_kernel<false>, dim3(a.B), dim3(nthreads), bytes, s, p, a, iters, L);
    }
    return hipGetLastError();
}

}  // namespace csk
