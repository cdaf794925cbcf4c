// Sketch y = Phi z (measurement equation, paper Sec. 3 / Sec. 8) with the
// operator generated on the fly: no entry of Phi is ever written to memory.
//
// Rademacher ensemble.  A workgroup owns RR rows of Phi and TB tokens; its 16
// wavefronts split the columns in tiles of 256.  Per tile, lane L < 2*RR draws the
// 128 sign bits of (row L % RR, call L / RR) with one Philox call; the words are
// handed to the other lanes with scalar lane reads.  Lane l owns columns
// l, l+64, l+128, l+192 of the tile, so the loads of z are coalesced and each value
// of z is reused for all RR rows from a register.  The RR*TB running sums per lane
// are reduced across the wavefront once at the end, then across wavefronts in LDS.
//
// Gaussian ensemble.  One wavefront per row and token chunk; a lane draws four
// normals per Philox call (Box-Muller) and applies them to one float4 of z.
#include "kernels.hpp"

namespace csk {

constexpr int SK_TB = 8;          // tokens per wavefront pass
constexpr int SK_WAVES = 4;       // rows per workgroup (Gaussian kernel)

constexpr int SR_RR = 4;          // rows per workgroup (Rademacher kernel)
constexpr int SR_TB = 8;          // tokens per workgroup
constexpr int SR_WAVES = 16;

__global__ __launch_bounds__(SR_WAVES * 64)
void sketch_rademacher_kernel(OpDesc op, const float* __restrict__ z, int B, float* __restrict__ y) {
    __shared__ float part[SR_WAVES][SR_RR * SR_TB];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row0 = blockIdx.x * SR_RR;
    const int t0 = blockIdx.y * SR_TB;
    const int nt = min(SR_TB, B - t0);
    const int n = op.n;
    float acc[SR_RR][SR_TB];
#pragma unroll
    for (int r = 0; r < SR_RR; ++r)
#pragma unroll
        for (int t = 0; t < SR_TB; ++t) acc[r][t] = 0.f;

    const int ntiles = (n + 255) >> 8;
    const uint32_t hi = (uint32_t)(lane >> 5);           // which half of the wave: selects the word pair
    const uint32_t sh = 31u - (uint32_t)(lane & 31);     // shift that moves this lane's bit to the sign position
    for (int tile = wave; tile < ntiles; tile += SR_WAVES) {
        // lane L < 2*RR: bits of row (row0 + L % RR), columns 128*(2*tile + L / RR) .. +127
        u32x4 bits;
        {
            const uint32_t r = (uint32_t)(lane % SR_RR), c = (uint32_t)(lane / SR_RR) & 1u;
            bits = rademacher_bits(op, (uint32_t)row0 + r, (uint32_t)(2 * tile) + c);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int col = (tile << 8) + 64 * q + lane;
            float zv[SR_TB];
#pragma unroll
            for (int t = 0; t < SR_TB; ++t) zv[t] = (col < n && t < nt) ? z[(size_t)(t0 + t) * n + col] : 0.f;
#pragma unroll
            for (int r = 0; r < SR_RR; ++r) {
                // column 64q + lane of the tile: call q/2, word 2*(q%2) + lane/32, bit lane%32
                const int src = (q >> 1) * SR_RR + r;
                const uint32_t wlo = __builtin_amdgcn_readlane(bits.w[2 * (q & 1)], src);
                const uint32_t whi = __builtin_amdgcn_readlane(bits.w[2 * (q & 1) + 1], src);
                const uint32_t sgn = ((hi ? whi : wlo) << sh) & 0x80000000u;
#pragma unroll
                for (int t = 0; t < SR_TB; ++t) acc[r][t] += __uint_as_float(__float_as_uint(zv[t]) ^ sgn);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < SR_RR; ++r)
#pragma unroll
        for (int t = 0; t < SR_TB; ++t) {
            const float s = wave_sum(acc[r][t]);
            if (lane == 0) part[wave][r * SR_TB + t] = s;
        }
    __syncthreads();
    if (threadIdx.x < SR_RR * SR_TB) {
        const int r = threadIdx.x / SR_TB, t = threadIdx.x % SR_TB;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < SR_WAVES; ++w) s += part[w][threadIdx.x];
        if (row0 + r < op.m && t < nt) y[(size_t)(t0 + t) * op.m + row0 + r] = s * op.scale;
    }
}

template <int TB, bool VEC>
__global__ __launch_bounds__(SK_WAVES * 64)
void sketch_gauss_kernel(OpDesc op, const float* __restrict__ z, int B, float* __restrict__ y) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * SK_WAVES + (threadIdx.x >> 6);
    const int t0 = blockIdx.y * TB;
    if (row >= op.m) return;
    const int nt = min(TB, B - t0);
    float acc[TB];
#pragma unroll
    for (int t = 0; t < TB; ++t) acc[t] = 0.f;
    const int ngroups = (op.n + 3) >> 2;
    for (int cg = lane; cg < ngroups; cg += 64) {
        float e[4];
        gauss4(op, (uint32_t)row, (uint32_t)cg, e);
        const int c0 = cg << 2;
        if (VEC && c0 + 4 <= op.n) {
#pragma unroll
            for (int t = 0; t < TB; ++t) {
                if (t < nt) {
                    const float4 v = *reinterpret_cast<const float4*>(z + (size_t)(t0 + t) * op.n + c0);
                    acc[t] += e[0] * v.x + e[1] * v.y + e[2] * v.z + e[3] * v.w;
                }
            }
        } else {
            for (int c = c0; c < min(c0 + 4, op.n); ++c)
                for (int t = 0; t < nt; ++t) acc[t] += e[c - c0] * z[(size_t)(t0 + t) * op.n + c];
        }
    }
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        const float s = wave_sum(acc[t]);
        if (lane == 0 && t < nt) y[(size_t)(t0 + t) * op.m + row] = s * op.scale;
    }
}

hipError_t launch_sketch(const OpDesc& op, const float* z, int B, float* y, hipStream_t s) {
    if (B <= 0) return hipSuccess;
    if (op.ens == 1) {
        dim3 grid((op.m + SR_RR - 1) / SR_RR, (B + SR_TB - 1) / SR_TB);
        hipLaunchKernelGGL(sketch_rademacher_kernel, grid, dim3(SR_WAVES * 64), 0, s, op, z, B, y);
    } else {
        dim3 grid((op.m + SK_WAVES - 1) / SK_WAVES, (B + SK_TB - 1) / SK_TB);
        const bool vec = (op.n & 3) == 0;   // float4 loads need 16-byte aligned rows of z
        if (vec) hipLaunchKernelGGL((sketch_gauss_kernel<SK_TB, true>), grid, dim3(SK_WAVES * 64), 0, s, op, z, B, y);
        else hipLaunchKernelGGL((sketch_gauss_kernel<SK_TB, false>), grid, dim3(SK_WAVES * 64), 0, s, op, z, B, y);
    }
    return hipGetLastError();
}

}  // namespace csk
