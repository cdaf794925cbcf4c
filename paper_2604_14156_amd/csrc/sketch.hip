// Sketch y = Phi z (measurement equation, paper Sec. 3 / Sec. 8) with the
// operator generated on the fly: no entry of Phi is ever written to memory.
//
// One wavefront owns one row of Phi and a chunk of TB tokens.  Rademacher: a lane
// draws 128 sign bits with one Philox call and applies them to 128 consecutive
// entries of z for each token of the chunk.  Gaussian: a lane draws four normals
// per call and applies them to one float4 of z per token.  Partial sums are
// reduced across the 64 lanes at the end.
#include "kernels.hpp"

namespace csk {

constexpr int SK_TB = 8;          // tokens per wavefront pass
constexpr int SK_WAVES = 4;       // rows per workgroup

template <int TB, bool VEC>
__global__ __launch_bounds__(SK_WAVES * 64)
void sketch_rademacher_kernel(OpDesc op, const float* __restrict__ z, int B, float* __restrict__ y) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * SK_WAVES + (threadIdx.x >> 6);
    const int t0 = blockIdx.y * TB;
    if (row >= op.m) return;
    const int nt = min(TB, B - t0);
    float acc[TB];
#pragma unroll
    for (int t = 0; t < TB; ++t) acc[t] = 0.f;
    const int ngroups = (op.n + 127) >> 7;
    for (int cg = lane; cg < ngroups; cg += 64) {
        const u32x4 bits = rademacher_bits(op, (uint32_t)row, (uint32_t)cg);
        const int c0 = cg << 7;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const uint32_t word = bits.w[w];
            const int cw = c0 + 32 * w;
            if (cw >= op.n) break;
            if (VEC && cw + 32 <= op.n) {
#pragma unroll
                for (int q4 = 0; q4 < 8; ++q4) {
#pragma unroll
                    for (int t = 0; t < TB; ++t) {
                        if (t < nt) {
                            const float4 v = *reinterpret_cast<const float4*>(z + (size_t)(t0 + t) * op.n + cw + 4 * q4);
                            const uint32_t sh = word >> (4 * q4);
                            // bit set -> minus: flip the sign bit of the float
                            acc[t] += __uint_as_float(__float_as_uint(v.x) ^ ((sh & 1u) << 31));
                            acc[t] += __uint_as_float(__float_as_uint(v.y) ^ ((sh & 2u) << 30));
                            acc[t] += __uint_as_float(__float_as_uint(v.z) ^ ((sh & 4u) << 29));
                            acc[t] += __uint_as_float(__float_as_uint(v.w) ^ ((sh & 8u) << 28));
                        }
                    }
                }
            } else {
                const int cend = min(cw + 32, op.n);
                for (int c = cw; c < cend; ++c) {
                    const uint32_t bit = (word >> (c - cw)) & 1u;
                    for (int t = 0; t < nt; ++t) {
                        const float v = z[(size_t)(t0 + t) * op.n + c];
                        acc[t] += bit ? -v : v;
                    }
                }
            }
        }
    }
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        const float s = wave_sum(acc[t]);
        if (lane == 0 && t < nt) y[(size_t)(t0 + t) * op.m + row] = s * op.scale;
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
    dim3 grid((op.m + SK_WAVES - 1) / SK_WAVES, (B + SK_TB - 1) / SK_TB);
    dim3 block(SK_WAVES * 64);
    const bool vec = (op.n & 3) == 0;   // float4 loads need 16-byte aligned rows of z
    if (op.ens == 1) {
        if (vec) hipLaunchKernelGGL((sketch_rademacher_kernel<SK_TB, true>), grid, block, 0, s, op, z, B, y);
        else hipLaunchKernelGGL((sketch_rademacher_kernel<SK_TB, false>), grid, block, 0, s, op, z, B, y);
    } else {
        if (vec) hipLaunchKernelGGL((sketch_gauss_kernel<SK_TB, true>), grid, block, 0, s, op, z, B, y);
        else hipLaunchKernelGGL((sketch_gauss_kernel<SK_TB, false>), grid, block, 0, s, op, z, B, y);
    }
    return hipGetLastError();
}

}  // namespace csk
