// Block orthogonal matching pursuit on the GPU (paper Sec. 8: "orthogonal matching
// pursuit over a constrained support dictionary"; support of exactly k units,
// Sec. 3 / Sec. 7).  One workgroup solves one sketch; the k rounds are sequential.
//
// The rounds run in the Gram domain.  With M = Phi Psi (Sec. 9), G = M^T M and
// c = M^T r, selecting atom a and orthogonalising it against the atoms already
// chosen gives a new orthonormal direction q; the vector d = M^T q obeys
//     d = (G[:,a] - sum_j d_j * d_j[a]) / nrm,    nrm^2 = G[a,a] - sum_j d_j[a]^2,
// the residual loses its component along q:  c <- c - (c[a]/nrm) d,
// and d_j[a_i] (j <= i) is the triangular factor R of the selected atoms (R^T R =
// G_SS), so the refit is a triangular solve.  This is the same greedy sequence and
// the same least-squares refit as the textbook algorithm, at O(N |S|) per round
// instead of O(N m).  After the last round the coefficients are refined once against
// the explicitly formed residual y - M_S alpha, which removes the squared condition
// number the Gram form would otherwise leave in the result.
#include "kernels.hpp"
#include <math.h>

namespace csk {

struct RecoverLayout {
    int off_corr, off_y, off_r, off_beta, off_alpha, off_gv, off_red, off_selcol, off_order, off_sel;
    int off_gram, off_D;      // -1: lives in global memory
    int total_floats;
};

static RecoverLayout make_layout(const Plan& p, int k, int lds_limit) {
    RecoverLayout L;
    const int N = p.N, m = p.op.m, K = k * p.rb;
    int o = 0;
    L.off_corr = o; o += N;
    L.off_y = o; o += m;
    L.off_r = o; o += m;
    L.off_beta = o; o += K;
    L.off_alpha = o; o += K;
    L.off_gv = o; o += K;
    L.off_red = o; o += 64;
    L.off_selcol = o; o += K;
    L.off_order = o; o += k;
    L.off_sel = o; o += p.G;
    o = (o + 3) & ~3;
    const long limit = lds_limit / 4 - 64;
    L.off_D = -1; L.off_gram = -1;
    if ((long)o + (long)K * N <= limit) { L.off_D = o; o += K * N; }
    o = (o + 3) & ~3;
    if ((long)o + (long)N * N <= limit) { L.off_gram = o; o += N * N; }
    L.total_floats = o;
    return L;
}

size_t recover_spill_floats(const Plan& p, int k, int lds_limit) {
    const RecoverLayout L = make_layout(p, k, lds_limit);
    return L.off_D < 0 ? (size_t)k * p.rb * p.N : 0;
}

struct Top2 { float s1; int i1; float s2; };

__device__ __forceinline__ Top2 top2_merge(const Top2& a, const Top2& b) {
    Top2 o;
    const bool a_wins = (a.s1 > b.s1) || (a.s1 == b.s1 && a.i1 <= b.i1);
    if (a_wins) { o.s1 = a.s1; o.i1 = a.i1; o.s2 = fmaxf(fmaxf(a.s2, b.s2), b.s1); }
    else        { o.s1 = b.s1; o.i1 = b.i1; o.s2 = fmaxf(fmaxf(a.s2, b.s2), a.s1); }
    return o;
}

__global__ void recover_kernel(Plan p, RecoverArgs a, RecoverLayout L) {
    extern __shared__ float lds[];
    const int tid = threadIdx.x, NT = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nwaves = NT >> 6;
    const int prob = blockIdx.x;
    const int N = p.N, m = p.op.m, rb = p.rb, G = p.G, k = a.k, K = k * rb;

    float* corr = lds + L.off_corr;
    float* yv = lds + L.off_y;
    float* rv = lds + L.off_r;
    float* beta = lds + L.off_beta;
    float* alpha = lds + L.off_alpha;
    float* gv = lds + L.off_gv;
    float* red = lds + L.off_red;
    int* selcol = reinterpret_cast<int*>(lds + L.off_selcol);
    int* order = reinterpret_cast<int*>(lds + L.off_order);
    int* sel = reinterpret_cast<int*>(lds + L.off_sel);
    // generic pointers: the factor and the Gram matrix live in LDS when they fit
    float* D = L.off_D >= 0 ? lds + L.off_D : a.spill + (size_t)prob * a.spill_stride;
    const float* gram = p.gram;
    if (L.off_gram >= 0) {
        float* gl = lds + L.off_gram;
        for (int i = tid; i < N * N; i += NT) gl[i] = p.gram[i];
        gram = gl;
    }

    const float* y = a.y + (size_t)prob * m;
    int bad_local = 0;
    for (int i = tid; i < m; i += NT) {
        const float v = y[i];
        yv[i] = v;
        if (!isfinite(v)) bad_local = 1;
    }
    for (int g = tid; g < G; g += NT) sel[g] = 0;
    if (tid == 0) { red[60] = 1.0f; red[61] = 0.0f; }       // margin, bad flag
    __syncthreads();
    if (bad_local) red[61] = 1.0f;

    // c = M^T y, one wavefront per atom
    for (int c = wave; c < N; c += nwaves) {
        const float* col = p.Mt + (size_t)c * m;
        float s = 0.f;
        for (int i = lane; i < m; i += 64) s += col[i] * yv[i];
        s = wave_sum(s);
        if (lane == 0) corr[c] = s;
    }
    __syncthreads();

    for (int round = 0; round < k; ++round) {
        // ---- score every unselected unit, keep the best two
        Top2 t; t.s1 = -1.f; t.i1 = 0x7fffffff; t.s2 = -1.f;
        for (int g = tid; g < G; g += NT) {
            if (sel[g]) continue;
            float s = 0.f;
            if (p.weighted) {
                const float* W = p.W + (size_t)g * rb * rb;
                for (int r = 0; r < rb; ++r) {
                    float v = 0.f;
                    for (int c = 0; c <= r; ++c) v += W[r * rb + c] * corr[g * rb + c];
                    s += v * v;
                }
            } else {
                for (int c = 0; c < rb; ++c) { const float v = corr[g * rb + c]; s += v * v; }
            }
            if (!(s >= 0.f)) s = -1.f;                       // NaN never wins
            Top2 u; u.s1 = s; u.i1 = g; u.s2 = -1.f;
            t = top2_merge(t, u);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            Top2 o;
            o.s1 = __shfl_xor(t.s1, off, 64);
            o.i1 = __shfl_xor(t.i1, off, 64);
            o.s2 = __shfl_xor(t.s2, off, 64);
            t = top2_merge(t, o);
        }
        if (lane == 0) { red[wave * 3] = t.s1; red[wave * 3 + 1] = __int_as_float(t.i1); red[wave * 3 + 2] = t.s2; }
        __syncthreads();
        if (tid == 0) {
            Top2 b; b.s1 = red[0]; b.i1 = __float_as_int(red[1]); b.s2 = red[2];
            for (int w = 1; w < nwaves; ++w) {
                Top2 o; o.s1 = red[w * 3]; o.i1 = __float_as_int(red[w * 3 + 1]); o.s2 = red[w * 3 + 2];
                b = top2_merge(b, o);
            }
            int gs = b.i1;
            if (b.s1 < 0.f || gs >= G) {                     // nothing scored: take the first free unit
                gs = 0;
                while (gs < G && sel[gs]) ++gs;
                red[61] = 1.0f;
                red[60] = 0.0f;
            } else {
                const float s2 = fmaxf(b.s2, 0.f);
                const float mg = b.s1 > 0.f ? (b.s1 - s2) / b.s1 : 0.f;
                red[60] = fminf(red[60], mg);
            }
            sel[gs] = 1;
            order[round] = gs;
            red[62] = __int_as_float(gs);
        }
        __syncthreads();
        const int gstar = __float_as_int(red[62]);

        // ---- append the unit's rb atoms to the factor, one at a time
        for (int q = 0; q < rb; ++q) {
            const int col = gstar * rb + q;
            const int J = round * rb + q;
            const float* grow = gram + (size_t)col * N;
            for (int c = tid; c < N; c += NT) {
                float s = 0.f;
                for (int j = 0; j < J; ++j) s += D[(size_t)j * N + c] * D[(size_t)j * N + col];
                D[(size_t)J * N + c] = grow[c] - s;
            }
            __syncthreads();
            const float nrm2 = D[(size_t)J * N + col];
            const float ccol = corr[col];
            const float gdiag = grow[col];
            __syncthreads();
            float inv = 0.f;
            if (nrm2 > 1e-10f * gdiag && nrm2 > 0.f) inv = 1.0f / sqrtf(nrm2);
            const float bt = ccol * inv;
            for (int c = tid; c < N; c += NT) {
                const float dv = D[(size_t)J * N + c] * inv;
                D[(size_t)J * N + c] = dv;
                corr[c] -= bt * dv;
            }
            if (tid == 0) {
                beta[J] = bt;
                selcol[J] = col;
                if (inv == 0.f) red[61] = 1.0f;
            }
            __syncthreads();
        }
    }

    // ---- R alpha = beta, R[j][i] = D[j][selcol[i]] (upper triangular), back substitution
    auto solve_upper = [&](float* rhs, float* out) {
        for (int i = K - 1; i >= 0; --i) {
            const float rii = D[(size_t)i * N + selcol[i]];
            const float v = rii > 0.f ? rhs[i] / rii : 0.f;
            __syncthreads();
            if (tid == 0) out[i] = v;
            for (int j = tid; j < i; j += NT) rhs[j] -= D[(size_t)j * N + selcol[i]] * v;
            __syncthreads();
        }
    };
    // R^T w = rhs (forward substitution), in place
    auto solve_lower_t = [&](float* rhs) {
        for (int i = 0; i < K; ++i) {
            const float rii = D[(size_t)i * N + selcol[i]];
            const float v = rii > 0.f ? rhs[i] / rii : 0.f;
            __syncthreads();
            if (tid == 0) rhs[i] = v;
            for (int l = i + 1 + tid; l < K; l += NT) rhs[l] -= D[(size_t)i * N + selcol[l]] * v;
            __syncthreads();
        }
    };
    solve_upper(beta, alpha);

    // ---- explicit residual r = y - M_S alpha
    for (int i = tid; i < m; i += NT) {
        float s = yv[i];
        for (int j = 0; j < K; ++j) s -= alpha[j] * p.Mt[(size_t)selcol[j] * m + i];
        rv[i] = s;
    }
    __syncthreads();
    // ---- one step of refinement: solve (R^T R) delta = M_S^T r
    for (int j = wave; j < K; j += nwaves) {
        const float* col = p.Mt + (size_t)selcol[j] * m;
        float s = 0.f;
        for (int i = lane; i < m; i += 64) s += col[i] * rv[i];
        s = wave_sum(s);
        if (lane == 0) gv[j] = s;
    }
    __syncthreads();
    solve_lower_t(gv);
    solve_upper(gv, beta);                                   // beta now holds delta
    for (int j = tid; j < K; j += NT) alpha[j] += beta[j];
    float ss = 0.f;
    for (int i = tid; i < m; i += NT) {
        float s = rv[i];
        for (int j = 0; j < K; ++j) s -= beta[j] * p.Mt[(size_t)selcol[j] * m + i];
        ss += s * s;
    }
    ss = wave_sum(ss);
    __syncthreads();
    if (lane == 0) red[wave] = ss;
    __syncthreads();

    // ---- outputs: ascending support, coefficients in that order
    const bool bad = red[61] != 0.f;
    for (int qi = tid; qi < k; qi += NT) {
        const int g = order[qi];
        int rank = 0;
        for (int o = 0; o < k; ++o) rank += order[o] < g;
        a.support[(size_t)prob * k + rank] = g;
        if (a.coef)
            for (int c = 0; c < rb; ++c) a.coef[(size_t)prob * K + rank * rb + c] = alpha[qi * rb + c];
    }
    if (tid == 0) {
        float tot = 0.f;
        for (int w = 0; w < nwaves; ++w) tot += red[w];
        if (a.resid) a.resid[prob] = bad ? __int_as_float(0x7fc00000) : sqrtf(tot);
        if (a.margin) a.margin[prob] = bad ? 0.f : red[60];
    }
}

hipError_t launch_recover(const Plan& p, const RecoverArgs& a, int lds_limit, hipStream_t s) {
    if (a.B <= 0) return hipSuccess;
    const RecoverLayout L = make_layout(p, a.k, lds_limit);
    int nt = 256;
    if (p.N > 256) nt = 512;
    if (p.N > 512) nt = 1024;
    const size_t bytes = (size_t)L.total_floats * 4;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(recover_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(recover_kernel, dim3(a.B), dim3(nt), bytes, s, p, a, L);
    return hipGetLastError();
}

}  // namespace csk
