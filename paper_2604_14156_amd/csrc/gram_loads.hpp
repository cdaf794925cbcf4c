// Start-up loads shared by the Gram-domain recovery kernels that work on one sketch per
// workgroup: the sketch into LDS, the Gram matrix into LDS (optional) and c0 = M^T y, one
// atom per thread.  Every independent global load is issued before the first wait.
#pragma once
#include "kernels.hpp"

namespace csk {

// yv: LDS [m]; gram_l: LDS [N*N] (GRAM_LDS only); stage: LDS scratch of 4 * blockDim.x floats.
// Returns c0 of atom `tid` (0 for tid >= N).  `bad` is set (workgroup-uniform) when the sketch
// holds a non-finite value.  Ends with a workgroup barrier after which yv, gram_l are complete
// and `stage` is free again.
template <bool GRAM_LDS>
__device__ __forceinline__ float load_sketch_gram_c0(const Plan& p, const float* __restrict__ y, float* yv,
                                                     float* gram_l, float* stage, int& bad) {
    const int tid = threadIdx.x, NT = blockDim.x;
    const int N = p.N, m = p.op.m;
    float yreg = (tid < m) ? y[tid] : 0.f;
    constexpr int GU = 16;
    const int n4 = (N * N) >> 2;
    float4 greg[GU];
    if (GRAM_LDS) {
        const float4* src = reinterpret_cast<const float4*>(p.gram);
#pragma unroll
        for (int u = 0; u < GU; ++u) {
            const int idx = u * NT + tid;
            greg[u] = idx < n4 ? src[idx] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    // slices of M^T y: a thread takes four adjacent atoms and a contiguous range of rows
    const bool vec4 = (N & 3) == 0;
    const int ncg = vec4 ? (N >> 2) : N;
    const int parts = NT / ncg > 0 ? NT / ncg : 1;
    const int cg = tid % ncg, part = tid / ncg;
    const int rows_per = (m + parts - 1) / parts;
    const int i0 = part * rows_per, i1 = part < parts ? min(m, i0 + rows_per) : i0;
    constexpr int MU = 8;
    float4 mreg[MU];
    if (vec4) {
        const float4* mr = reinterpret_cast<const float4*>(p.Mr) + cg;
#pragma unroll
        for (int u = 0; u < MU; ++u)
            mreg[u] = (i0 + u < i1) ? mr[(size_t)(i0 + u) * ncg] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    int mybad = !isfinite(yreg);
    if (tid < m) yv[tid] = yreg;
    for (int i = tid + NT; i < m; i += NT) {            // only when m exceeds the workgroup size
        const float v = y[i];
        yv[i] = v;
        if (!isfinite(v)) mybad = 1;
    }
    if (GRAM_LDS) {
        float4* dst = reinterpret_cast<float4*>(gram_l);
#pragma unroll
        for (int u = 0; u < GU; ++u) {
            const int idx = u * NT + tid;
            if (idx < n4) dst[idx] = greg[u];
        }
        const float4* src = reinterpret_cast<const float4*>(p.gram);
        for (int base = GU * NT; base < n4; base += NT) {     // Gram matrices beyond the first batch
            const int idx = base + tid;
            if (idx < n4) dst[idx] = src[idx];
        }
        for (int i = (n4 << 2) + tid; i < N * N; i += NT) gram_l[i] = p.gram[i];
    }
    bad = __syncthreads_or(mybad | bad);
    if (vec4) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        const float4* mr = reinterpret_cast<const float4*>(p.Mr) + cg;
        for (int ib = i0; ib < i1; ib += MU) {
            if (ib != i0) {
#pragma unroll
                for (int u = 0; u < MU; ++u)
                    mreg[u] = (ib + u < i1) ? mr[(size_t)(ib + u) * ncg] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int u = 0; u < MU; ++u)
                if (ib + u < i1) {
                    const float yy = yv[ib + u];
                    acc.x += mreg[u].x * yy; acc.y += mreg[u].y * yy; acc.z += mreg[u].z * yy; acc.w += mreg[u].w * yy;
                }
        }
        if (part < parts) reinterpret_cast<float4*>(stage)[part * ncg + cg] = acc;
    } else {
        float acc = 0.f;
#pragma unroll 8
        for (int i = i0; i < i1; ++i) acc += p.Mr[(size_t)i * N + cg] * yv[i];
        if (part < parts) stage[part * N + cg] = acc;
    }
    __syncthreads();
    float c0 = 0.f;
    if (tid < N) for (int q = 0; q < parts; ++q) c0 += stage[q * N + tid];
    __syncthreads();
    return c0;
}

}  // namespace csk
