// Small dense linear algebra on one wavefront, for the refits of the recovery kernels:
// Cholesky factor of a Gram sub-matrix G_SS (at most 64 units), appending one unit to it,
// and the two triangular solves.  The factor lives in LDS, one row per unit with a row
// stride chosen by the caller (odd strides keep column reads conflict free); lane j owns
// unit j of the list.  All lanes of the wavefront must call these together.
#pragma once
#include "common.hpp"

namespace csk {

// L L^T = G_SS + ridge I for the K units S[0..K).  Returns 1 if a pivot was not positive
// (repeated or linearly dependent units), else 0.
__device__ __forceinline__ int wave_cholesky(const float* gram, int N, const int* S, int K, float ridge,
                                             float* Lf, int LS, int lane) {
    int bad = 0;
    for (int i = 0; i < K; ++i) {
        const int si = S[i];
        if (lane >= i && lane < K) {
            const int sj = S[lane];
            float s = gram[(size_t)si * N + sj] + (lane == i ? ridge : 0.f);
            for (int t = 0; t < i; ++t) s -= Lf[lane * LS + t] * Lf[i * LS + t];
            Lf[lane * LS + i] = s;                  // un-normalised; row i's own entry is the pivot
        }
        __builtin_amdgcn_wave_barrier();
        const float piv = Lf[i * LS + i];
        const float inv = piv > 0.f ? __builtin_amdgcn_rsqf(piv) : 0.f;
        if (!(piv > 0.f)) bad = 1;
        __builtin_amdgcn_wave_barrier();
        if (lane >= i && lane < K) Lf[lane * LS + i] *= inv;          // L[i][i] = sqrt(piv), L[j][i] /= sqrt(piv)
        __builtin_amdgcn_wave_barrier();
    }
    return bad;
}

// Row K of the factor for a new unit `a` appended to S[0..K): L[K][0..K) = L^{-1} G[S, a] and the new
// diagonal entry.  Returns 1 if the new pivot was not positive.
__device__ __forceinline__ int wave_cholesky_append(const float* gram, int N, const int* S, int K, int a,
                                                    float* Lf, int LS, int lane) {
    float rhs = lane < K ? gram[(size_t)a * N + S[lane]] : 0.f;
    for (int i = 0; i < K; ++i) {
        const float lii = Lf[i * LS + i];
        const float xi = lii > 0.f ? readlane_f32(rhs, i) / lii : 0.f;
        if (lane == i) rhs = xi;
        if (lane > i && lane < K) rhs -= Lf[lane * LS + i] * xi;
    }
    const float piv = gram[(size_t)a * N + a] - wave_sum(lane < K ? rhs * rhs : 0.f);
    if (lane < K) Lf[K * LS + lane] = rhs;
    if (lane == K) Lf[K * LS + K] = piv > 0.f ? sqrtf(piv) : 0.f;
    __builtin_amdgcn_wave_barrier();
    return piv > 0.f ? 0 : 1;
}

// Solves L L^T x = rhs (forward, then backward substitution); lane i passes rhs_i and gets x_i.
__device__ __forceinline__ float wave_cholesky_solve(const float* Lf, int LS, int K, float rhs, int lane) {
    for (int i = 0; i < K; ++i) {
        const float lii = Lf[i * LS + i];
        const float xi = lii > 0.f ? readlane_f32(rhs, i) / lii : 0.f;
        if (lane == i) rhs = xi;
        if (lane > i && lane < K) rhs -= Lf[lane * LS + i] * xi;
    }
    for (int i = K - 1; i >= 0; --i) {
        const float lii = Lf[i * LS + i];
        const float xi = lii > 0.f ? readlane_f32(rhs, i) / lii : 0.f;
        if (lane == i) rhs = xi;
        if (lane < i) rhs -= Lf[i * LS + lane] * xi;
    }
    return rhs;
}

}  // namespace csk
