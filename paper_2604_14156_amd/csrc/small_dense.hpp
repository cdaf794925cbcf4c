// Small dense linear algebra on one wavefront, for the refits of the recovery kernels:
// Cholesky factor of a Gram sub-matrix G_SS (at most 64 units), appending one unit to it,
// and the two triangular solves.  Lane j owns unit j of the list.  All lanes of the wavefront
// must call these together.
//
// Storage of the factor (LDS): row i of L at Lf + i * SD_LS, SD_LS = 65 floats (odd: column reads
// are conflict free).  Only the strictly lower triangle is stored in columns 0..63; the diagonal
// and everything above it are kept at zero, and column 64 of row i holds 1 / L[i][i].  With the
// zeros in place the substitutions need no lane masks: every step is one scalar lane read, one
// multiply and one multiply-add on all lanes.
//
// These are latency chains of K steps, so nothing that can be fetched ahead sits inside a chain:
// the factorisation keeps the matrix in registers (lane j = row j) and hands the pivot column
// round through a 64-float LDS buffer, and the substitutions fetch eight columns / rows of the
// factor ahead of the eight dependent steps that use them.
#pragma once
#include "common.hpp"

namespace csk {

constexpr int SD_MAXK = 64;
constexpr int SD_LS = SD_MAXK + 1;

// L L^T = G_SS + ridge I for the K units S[0..K) (S in LDS, K <= 64).  Returns 1 if a pivot was not
// positive (repeated or linearly dependent units), else 0.  Rows K.. of Lf are not touched.
// colbuf: 64 floats of LDS scratch, 16-byte aligned.
// Right-looking elimination: at step i register r of lane j holds entry (j, i + r), i.e. every step
// shifts the row down by one register while it applies the update, so register indices are
// compile-time constants although the step loop is rolled.
__device__ __forceinline__ int wave_cholesky(const float* gram, int N, const int* S, int K, float ridge,
                                             float* Lf, float* colbuf, int lane) {
    float a[SD_MAXK];
    const int sj = S[lane < K ? lane : 0];
#pragma unroll
    for (int t = 0; t < SD_MAXK; ++t) {
        const int st = S[t < K ? t : 0];
        a[t] = (t < K ? gram[(size_t)sj * N + st] : 0.f) + (t == lane ? ridge : 0.f);
    }
    int bad = 0;
#pragma unroll 1
    for (int i = 0; i < K; ++i) {
        const float piv = readlane_f32(a[0], i);
        if (!(piv > 0.f)) bad = 1;
        const float inv = piv > 0.f ? __builtin_amdgcn_rsqf(piv) : 0.f;
        const float l = a[0] * inv;                     // lane j > i: L[j][i]
        if (lane < K) Lf[lane * SD_LS + i] = lane > i ? l : 0.f;
        if (lane == i) Lf[i * SD_LS + SD_MAXK] = inv;
        // column entries of rows i+1.. in colbuf[0..]: the update of column i + r needs L[i + r][i]
        if (lane > i) colbuf[lane - i - 1] = l;
        __builtin_amdgcn_wave_barrier();
        const int rem = K - i;                          // columns i .. K-1 are registers 0 .. rem-1
        // the whole buffer is fetched before the first use: one LDS latency per step, not one per chunk
        float4 cq[SD_MAXK / 4];
#pragma unroll
        for (int c = 0; c < SD_MAXK / 4; ++c) cq[c] = *reinterpret_cast<const float4*>(colbuf + 4 * c);
#pragma unroll
        for (int r0 = 1; r0 < SD_MAXK; r0 += 8) {
            if (r0 < rem) {                             // uniform
                const float4 c0 = cq[(r0 - 1) / 4], c1 = cq[(r0 - 1) / 4 + 1];
                const float cv[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int r = r0 + u;
                    if (r < SD_MAXK) a[r - 1] = a[r] - l * cv[u];       // meaningful for rows >= column only
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    // columns K.. of the rows just built are above the diagonal of any factor grown from this one
    if (lane < K)
        for (int t = K; t < SD_MAXK; ++t) Lf[lane * SD_LS + t] = 0.f;
    __builtin_amdgcn_wave_barrier();
    return bad;
}

// Forward substitution L z = rhs; lane i passes rhs_i and gets z_i.
__device__ __forceinline__ float wave_forward(const float* Lf, int K, float rhs, int lane) {
    const int row = (lane < K ? lane : 0) * SD_LS;
    for (int i0 = 0; i0 < K; i0 += 8) {
        float col[8], di[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = min(i0 + u, K - 1);
            col[u] = Lf[row + i];                       // zero for lanes <= i
            di[u] = i0 + u < K ? Lf[i * SD_LS + SD_MAXK] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float zi = readlane_f32(rhs, min(i0 + u, SD_MAXK - 1)) * di[u];      // steps past K add zero
            rhs -= col[u] * zi;
        }
    }
    return rhs * Lf[row + SD_MAXK];
}

// Backward substitution L^T x = z; lane i passes z_i and gets x_i.
__device__ __forceinline__ float wave_backward(const float* Lf, int K, float rhs, int lane) {
    const int lc = lane < K ? lane : 0;
    for (int i0 = K - 1; i0 >= 0; i0 -= 8) {
        float row[8], di[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = max(i0 - u, 0);
            row[u] = Lf[i * SD_LS + lc];                // zero for lanes >= i
            di[u] = i0 - u >= 0 ? Lf[i * SD_LS + SD_MAXK] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float xi = readlane_f32(rhs, max(i0 - u, 0)) * di[u];                 // steps below 0 add zero
            rhs -= row[u] * xi;
        }
    }
    return rhs * Lf[lc * SD_LS + SD_MAXK];
}

// Solves L L^T x = rhs; lane i passes rhs_i and gets x_i.
__device__ __forceinline__ float wave_cholesky_solve(const float* Lf, int K, float rhs, int lane) {
    return wave_backward(Lf, K, wave_forward(Lf, K, rhs, lane), lane);
}

// Row K of the factor for a new unit `a` appended to S[0..K), K < 64: L[K][0..K) = L^{-1} G[S, a] and
// the new diagonal entry.  Returns 1 if the new pivot was not positive.  `row`, if given, receives
// L[K][lane] for lane < K (0 elsewhere).
__device__ __forceinline__ int wave_cholesky_append(const float* gram, int N, const int* S, int K, int a,
                                                    float* Lf, int lane, float* row = nullptr) {
    float rhs = lane < K ? gram[(size_t)a * N + S[lane]] : 0.f;
    rhs = wave_forward(Lf, K, rhs, lane);
    if (lane >= K) rhs = 0.f;
    if (row) *row = rhs;
    const float piv = gram[(size_t)a * N + a] - wave_sum(rhs * rhs);
    const bool ok = piv > 0.f;
    Lf[K * SD_LS + lane] = rhs;                         // zero on and above the diagonal
    if (lane == K) Lf[K * SD_LS + SD_MAXK] = ok ? __builtin_amdgcn_rsqf(piv) : 0.f;
    __builtin_amdgcn_wave_barrier();
    return ok ? 0 : 1;
}

}  // namespace csk
