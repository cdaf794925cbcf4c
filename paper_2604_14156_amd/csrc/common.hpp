// Device-side helpers shared by the kernels: Philox4x32-10, the operator's entry
// function, bf16 conversion, wavefront (64-lane) reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "op_desc.hpp"

#define CS_WAVE 64

namespace csk {

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies
// with key injection; the key advances by two Weyl constants between rounds.
// ---------------------------------------------------------------------------
struct u32x4 { uint32_t w[4]; };

__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    u32x4 o; o.w[0] = c0; o.w[1] = c1; o.w[2] = c2; o.w[3] = c3;
    return o;
}


// 128 sign bits of row `row`, column group `cg` (columns 128*cg .. 128*cg+127).
__device__ __forceinline__ u32x4 rademacher_bits(const OpDesc& op, uint32_t row, uint32_t cg) {
    return philox4x32_10(cg, row, op.stream, 1u, op.k0, op.k1);
}

// Subsampled randomised Hadamard ensemble: entry (i, c) = d_c * (-1)^popcount(r_i & c), with the sign
// d_c = Rademacher bit of column c under counter (c / 128, 0, stream, 2) and the row map
// r_i = perm(i), a bijection of [0, 2^nbits) keyed by the Philox call with counter (0, 1, stream, 2):
// two rounds of (multiply by an odd word, add a word, fold the upper half onto the lower).
struct SrhtRows { uint32_t a1, c1, a2, c2, mask; int fold; };
__device__ __forceinline__ SrhtRows srht_rows_key(const OpDesc& op) {
    const u32x4 w = philox4x32_10(0u, 1u, op.stream, 2u, op.k0, op.k1);
    SrhtRows r;
    r.a1 = w.w[0] | 1u; r.c1 = w.w[1]; r.a2 = w.w[2] | 1u; r.c2 = w.w[3];
    r.mask = op.nbits >= 32 ? 0xFFFFFFFFu : ((1u << op.nbits) - 1u);
    r.fold = (op.nbits + 1) >> 1;
    return r;
}
__device__ __forceinline__ uint32_t srht_row(const SrhtRows& k, uint32_t i) {
    uint32_t x = (i * k.a1 + k.c1) & k.mask;
    x ^= x >> k.fold;
    x = (x * k.a2 + k.c2) & k.mask;
    x ^= x >> k.fold;
    return x;
}
// 128 sign bits d_c of column group `cg`
__device__ __forceinline__ u32x4 srht_sign_bits(const OpDesc& op, uint32_t cg) {
    return philox4x32_10(cg, 0u, op.stream, 2u, op.k0, op.k1);
}

// ln(u) for u = (w+1)/2^32 in (0,1], accurate also when u is close to 1, where a
// plain float conversion of u would lose the distance to 1.
__device__ __forceinline__ float log_unit_open(uint32_t w) {
    const uint32_t dist = 0xFFFFFFFFu - w;            // 2^32 - (w+1), exact
    if (dist < (1u << 24)) return log1pf(-(float)dist * 2.3283064365386963e-10f);
    // (w+1)*2^-32 with w+1 formed in double to stay exact up to 2^32
    return logf((float)(((double)w + 1.0) * 2.3283064365386963e-10));
}

// The four Gaussian entries of row `row`, column group `cg` (columns 4*cg .. 4*cg+3).
__device__ __forceinline__ void gauss4(const OpDesc& op, uint32_t row, uint32_t cg, float e[4]) {
    const u32x4 o = philox4x32_10(cg, row, op.stream, 0u, op.k0, op.k1);
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const float rad = sqrtf(-2.0f * log_unit_open(o.w[2 * p]));
        // angle = 2*pi*u2; sincospif takes the argument in units of pi and reduces it exactly
        const float turns2 = (float)(((double)o.w[2 * p + 1] + 1.0) * 4.656612873077393e-10);  // 2*u2
        float s, c;
        sincospif(turns2, &s, &c);
        e[2 * p] = rad * c;
        e[2 * p + 1] = rad * s;
    }
}

// ---------------------------------------------------------------------------
// bf16 <-> fp32 on raw bits
// ---------------------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xFFFF0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {       // round to nearest even
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);   // NaN stays NaN
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// Eight consecutive elements as floats.
__device__ __forceinline__ void load8(const float* p, float v[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p);
    const float4 b = *reinterpret_cast<const float4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const uint16_t* p, float v[8]) {
    const uint4 a = *reinterpret_cast<const uint4*>(p);
    v[0] = bf16_lo(a.x); v[1] = bf16_hi(a.x); v[2] = bf16_lo(a.y); v[3] = bf16_hi(a.y);
    v[4] = bf16_lo(a.z); v[5] = bf16_hi(a.z); v[6] = bf16_lo(a.w); v[7] = bf16_hi(a.w);
}
__device__ __forceinline__ void store1(float* p, float v) { *p = v; }
__device__ __forceinline__ void store1(uint16_t* p, float v) { *p = f32_to_bf16(v); }
__device__ __forceinline__ float load1(const float* p) { return *p; }
__device__ __forceinline__ float load1(const uint16_t* p) { return bf16_to_f32(*p); }

// ---------------------------------------------------------------------------
// wavefront reductions (64 lanes) on the data-parallel-primitive lane crossbar:
// each step is one VALU instruction that reads a permuted copy of a register.
// A row is 16 lanes.  Steps: swap within pairs, swap pairs within quads, mirror
// within half rows, mirror within rows; afterwards every lane of a row holds the
// row's result, and the four rows are combined through scalar lane reads.
// ---------------------------------------------------------------------------
#define CS_DPP_QUAD_SWAP1 0xB1      /* quad_perm [1,0,3,2] */
#define CS_DPP_QUAD_SWAP2 0x4E      /* quad_perm [2,3,0,1] */
#define CS_DPP_HALF_MIRROR 0x141
#define CS_DPP_ROW_MIRROR 0x140

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float readlane_f32(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// sum over aligned groups of WIDTH lanes (WIDTH in {2,4,8,16,32,64}); every lane gets the result
template <int WIDTH>
__device__ __forceinline__ float group_sum(float v) {
    if (WIDTH >= 2) v += dpp_f32<CS_DPP_QUAD_SWAP1>(v);
    if (WIDTH >= 4) v += dpp_f32<CS_DPP_QUAD_SWAP2>(v);
    if (WIDTH >= 8) v += dpp_f32<CS_DPP_HALF_MIRROR>(v);
    if (WIDTH >= 16) v += dpp_f32<CS_DPP_ROW_MIRROR>(v);
    if (WIDTH == 32) v += __shfl_xor(v, 16, 64);
    if (WIDTH == 64) v = (readlane_f32(v, 0) + readlane_f32(v, 16)) + (readlane_f32(v, 32) + readlane_f32(v, 48));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) { return group_sum<64>(v); }
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_f32<CS_DPP_QUAD_SWAP1>(v));
    v = fmaxf(v, dpp_f32<CS_DPP_QUAD_SWAP2>(v));
    v = fmaxf(v, dpp_f32<CS_DPP_HALF_MIRROR>(v));
    v = fmaxf(v, dpp_f32<CS_DPP_ROW_MIRROR>(v));
    return fmaxf(fmaxf(readlane_f32(v, 0), readlane_f32(v, 16)), fmaxf(readlane_f32(v, 32), readlane_f32(v, 48)));
}

}  // namespace csk
