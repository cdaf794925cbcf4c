// Plan-time (cold) kernels: the effective sensing matrix M = Phi Psi of paper
// Sec. 9, its column Gram matrix, and the per-unit weights that turn a unit's
// correlations into the energy of the residual inside the unit's column space.
// Sums run in fp64 and are rounded once: these run once per (operator,
// dictionary) pair, never in the per-token loop.
#include "kernels.hpp"
#include "common.hpp"

namespace csk {

constexpr int CS_MAX_RB_WEIGHTED = 16;

// `hrow`: the Hadamard row of measurement `row` (Hadamard ensemble only)
__device__ __forceinline__ float phi_entry_unscaled(const OpDesc& op, uint32_t row, uint32_t hrow, uint32_t col) {
    if (op.ens == 2) {
        const u32x4 bits = srht_sign_bits(op, col >> 7);
        const uint32_t d = (bits.w[(col & 127u) >> 5] >> (col & 31u)) & 1u;
        return ((__popc(hrow & col) ^ d) & 1u) ? -1.f : 1.f;
    }
    if (op.ens == 1) {
        const u32x4 bits = rademacher_bits(op, row, col >> 7);
        const uint32_t bit = (bits.w[(col & 127u) >> 5] >> (col & 31u)) & 1u;
        return bit ? -1.f : 1.f;
    }
    float e[4];
    gauss4(op, row, col >> 2, e);
    return e[col & 3u];
}

// Mt[g*rb + j][i] = scale * sum_t e(i, g*b + t) * psi[g][t][j]   (psi == nullptr: identity, rb == b)
__global__ void build_atoms_kernel(Plan p, const float* __restrict__ psi) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;    // measurement row
    const int g = blockIdx.y;
    if (i >= p.op.m) return;
    const int m = p.op.m;
    const uint32_t hrow = p.op.ens == 2 ? srht_row(srht_rows_key(p.op), (uint32_t)i) : 0u;
    if (psi == nullptr) {
        for (int t = 0; t < p.b; ++t)
            p.Mt[(size_t)(g * p.b + t) * m + i] = phi_entry_unscaled(p.op, i, hrow, g * p.b + t) * p.op.scale;
        return;
    }
    for (int j0 = 0; j0 < p.rb; j0 += 4) {
        double acc[4] = {0.0, 0.0, 0.0, 0.0};
        for (int t = 0; t < p.b; ++t) {
            const double e = (double)phi_entry_unscaled(p.op, i, hrow, g * p.b + t);
            for (int j = 0; j < 4; ++j)
                if (j0 + j < p.rb) acc[j] += e * (double)psi[((size_t)g * p.b + t) * p.rb + j0 + j];
        }
        for (int j = 0; j < 4; ++j)
            if (j0 + j < p.rb) p.Mt[(size_t)(g * p.rb + j0 + j) * m + i] = (float)(acc[j] * (double)p.op.scale);
    }
}

// Mr[i][c] = Mt[c][i]
__global__ void transpose_atoms_kernel(Plan p) {
    __shared__ float tile[16][17];
    const int c0 = blockIdx.x * 16, i0 = blockIdx.y * 16;
    const int ty = threadIdx.y, tx = threadIdx.x;
    if (c0 + ty < p.N && i0 + tx < p.op.m) tile[ty][tx] = p.Mt[(size_t)(c0 + ty) * p.op.m + i0 + tx];
    __syncthreads();
    if (i0 + ty < p.op.m && c0 + tx < p.N) p.Mr[(size_t)(i0 + ty) * p.N + c0 + tx] = tile[tx][ty];
}

// gram[a][c] = <Mt[a], Mt[c]>
__global__ void gram_kernel(Plan p) {
    __shared__ float ta[16][17], tc[16][17];
    const int a0 = blockIdx.y * 16, c0 = blockIdx.x * 16;
    const int ty = threadIdx.y, tx = threadIdx.x;
    double acc = 0.0;
    for (int i0 = 0; i0 < p.op.m; i0 += 16) {
        ta[ty][tx] = (a0 + ty < p.N && i0 + tx < p.op.m) ? p.Mt[(size_t)(a0 + ty) * p.op.m + i0 + tx] : 0.f;
        tc[ty][tx] = (c0 + ty < p.N && i0 + tx < p.op.m) ? p.Mt[(size_t)(c0 + ty) * p.op.m + i0 + tx] : 0.f;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 16; ++i) acc += (double)ta[ty][i] * (double)tc[tx][i];
        __syncthreads();
    }
    if (a0 + ty < p.N && c0 + tx < p.N) p.gram[(size_t)(a0 + ty) * p.N + c0 + tx] = (float)acc;
}

// W[g] = inverse of the Cholesky factor of the unit's rb x rb Gram block, so that
// || W[g] c_g ||^2 = c_g^T (M_g^T M_g)^{-1} c_g = energy of r in span(M_g) when c_g = M_g^T r.
__global__ void unit_weights_kernel(Plan p) {
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= p.G) return;
    const int rb = p.rb;
    double L[CS_MAX_RB_WEIGHTED][CS_MAX_RB_WEIGHTED];
    for (int a = 0; a < rb; ++a)
        for (int c = 0; c <= a; ++c) {
            double s = (double)p.gram[(size_t)(g * rb + a) * p.N + g * rb + c];
            for (int t = 0; t < c; ++t) s -= L[a][t] * L[c][t];
            L[a][c] = (a == c) ? sqrt(fmax(s, 0.0)) : (L[c][c] > 0.0 ? s / L[c][c] : 0.0);
        }
    // invert the lower-triangular factor column by column
    float* W = p.W + (size_t)g * rb * rb;
    for (int c = 0; c < rb; ++c)
        for (int a = 0; a < rb; ++a) {
            double v = 0.0;
            if (a >= c) {
                double s = (a == c) ? 1.0 : 0.0;
                for (int t = c; t < a; ++t) s -= L[a][t] * (double)W[t * rb + c];
                v = L[a][a] > 0.0 ? s / L[a][a] : 0.0;
            }
            W[a * rb + c] = (float)v;
        }
}

hipError_t launch_plan_build(const Plan& p, const float* psi, hipStream_t s) {
    {
        dim3 block(128), grid((p.op.m + 127) / 128, p.G);
        hipLaunchKernelGGL(build_atoms_kernel, grid, block, 0, s, p, psi);
    }
    {
        dim3 block(16, 16), grid((p.N + 15) / 16, (p.op.m + 15) / 16);
        hipLaunchKernelGGL(transpose_atoms_kernel, grid, block, 0, s, p);
    }
    {
        dim3 block(16, 16), grid((p.N + 15) / 16, (p.N + 15) / 16);
        hipLaunchKernelGGL(gram_kernel, grid, block, 0, s, p);
    }
    if (p.weighted) {
        dim3 block(64), grid((p.G + 63) / 64);
        hipLaunchKernelGGL(unit_weights_kernel, grid, block, 0, s, p);
    }
    return hipGetLastError();
}

}  // namespace csk
