// Sketch y = Phi z (measurement equation, paper Sec. 3 / Sec. 8) with the
// operator generated on the fly: no entry of Phi is ever written to memory.
//
// Rademacher ensemble.  A workgroup owns RR rows of Phi and TB tokens; its 16
// wavefronts split the columns in tiles of 256 (wave w takes tiles w, w+16, ...).  One Philox
// pass of a wave draws the sign bits of all its tiles at once: 2*RR lanes per tile, lane = (tile,
// call, row), 128 bits each; the words are handed to the other lanes with scalar lane reads.
// Lane l owns columns l, l+64, l+128, l+192 of a tile, so the loads of z are coalesced and each
// value of z is reused for all RR rows from a register; an entry costs one multiply-add with
// +-1.0.  The RR*TB running sums per lane are reduced across the wavefront once at the end, then
// across wavefronts in LDS.
//
// Gaussian ensemble.  One wavefront per row and token chunk; a lane draws four
// normals per Philox call (Box-Muller) and applies them to one float4 of z.
//
// Subsampled randomised Hadamard ensemble.  y = (1/sqrt(m)) (H (d * z))[r_i]: one workgroup per
// token holds the signed, zero-padded vector in LDS and runs the fast Walsh-Hadamard transform
// on it, four butterfly levels per pass with the sixteen values of a group in registers (the
// levels of the transform commute, so the passes simply walk over the index bits), then reads
// the m selected entries.  n' log2 n' additions per token instead of m n.
#include "kernels.hpp"
#include "common.hpp"

namespace csk {

constexpr int SK_TB = 8;          // tokens per wavefront pass
constexpr int SK_WAVES = 4;       // rows per workgroup (Gaussian kernel)

constexpr int SR_WAVES = 16;

// Several operators of one shape in a launch: blockIdx.z picks the operator, whose Philox key and
// stream come from this table (passed by value); its vectors and sketches follow those of the
// previous operator in z and y.
constexpr int SK_MAX_OPS = 32;
struct OpKeys { uint32_t k0[SK_MAX_OPS], k1[SK_MAX_OPS], stream[SK_MAX_OPS]; };

__device__ __forceinline__ void pick_operator(OpDesc& op, const OpKeys& keys) {
    const int j = blockIdx.z;
    op.k0 = keys.k0[j]; op.k1 = keys.k1[j]; op.stream = keys.stream[j];
}

// RR rows of Phi and TB tokens per workgroup.  The kernel is a short latency chain (one Philox
// call, one round trip for z, the reductions), so the launcher picks the smallest RR that still
// gives every compute unit a workgroup.
template <int RR, int TB>
__global__ __launch_bounds__(SR_WAVES * 64)
void sketch_rademacher_kernel(OpDesc op, OpKeys keys, const float* __restrict__ z, int B, float* __restrict__ y) {
    __shared__ float part[SR_WAVES][RR * TB];
    pick_operator(op, keys);
    z += (size_t)blockIdx.z * B * op.n;
    y += (size_t)blockIdx.z * B * op.m;
    constexpr int PER = 2 * RR;              // lanes that draw the bits of one 256-column tile
    constexpr int CH = 64 / PER;             // tiles covered by one Philox pass of the wave
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row0 = blockIdx.x * RR;
    const int t0 = blockIdx.y * TB;
    const int nt = min(TB, B - t0);
    const int n = op.n;
    float acc[RR][TB];
#pragma unroll
    for (int r = 0; r < RR; ++r)
#pragma unroll
        for (int t = 0; t < TB; ++t) acc[r][t] = 0.f;

    const int ntiles = (n + 255) >> 8;
    const uint32_t hi = (uint32_t)(lane >> 5);           // which half of the wave: selects the word pair
    const uint32_t sh = 31u - (uint32_t)(lane & 31);     // shift that moves this lane's bit to the sign position
    // this wave's tiles are wave, wave + 16, wave + 32, ...; one Philox pass draws the bits of CH of them:
    // lane L holds row (row0 + L % RR), call (L / RR) % 2 of tile number L / PER of the pass
    for (int j0 = 0; wave + j0 * SR_WAVES < ntiles; j0 += CH) {
        u32x4 bits;
        {
            const uint32_t l = (uint32_t)(lane % PER);
            const uint32_t tl = (uint32_t)(wave + (j0 + lane / PER) * SR_WAVES);
            bits = rademacher_bits(op, (uint32_t)row0 + l % RR, 2u * tl + l / RR);
        }
#pragma unroll 1
        for (int jj = 0; jj < CH; ++jj) {
            const int tile = wave + (j0 + jj) * SR_WAVES;
            if (tile >= ntiles) break;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = (tile << 8) + 64 * q + lane;
                float zv[TB];
#pragma unroll
                for (int t = 0; t < TB; ++t) zv[t] = (col < n && t < nt) ? z[(size_t)(t0 + t) * n + col] : 0.f;
#pragma unroll
                for (int r = 0; r < RR; ++r) {
                    // column 64q + lane of the tile: call q/2, word 2*(q%2) + lane/32, bit lane%32
                    const int src = jj * PER + (q >> 1) * RR + r;
                    const uint32_t wlo = __builtin_amdgcn_readlane(bits.w[2 * (q & 1)], src);
                    const uint32_t whi = __builtin_amdgcn_readlane(bits.w[2 * (q & 1) + 1], src);
                    // +-1.0 built from the sign bit; one multiply-add per entry (the product is exact)
                    const float pm = __uint_as_float((((hi ? whi : wlo) << sh) & 0x80000000u) | 0x3F800000u);
#pragma unroll
                    for (int t = 0; t < TB; ++t) acc[r][t] = fmaf(pm, zv[t], acc[r][t]);
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < RR; ++r)
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            const float s = wave_sum(acc[r][t]);
            if (lane == 0) part[wave][r * TB + t] = s;
        }
    __syncthreads();
    if (threadIdx.x < RR * TB) {
        const int r = threadIdx.x / TB, t = threadIdx.x % TB;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < SR_WAVES; ++w) s += part[w][threadIdx.x];
        if (row0 + r < op.m && t < nt) y[(size_t)(t0 + t) * op.m + row0 + r] = s * op.scale;
    }
}

// Rademacher ensemble on the matrix cores, for launches that sketch many operators at once.
// y = Phi z is a dense contraction once 16 tokens share the rows: a workgroup owns 16 rows of Phi and 16
// tokens, its 16 waves split the columns in chunks of 128 (one Philox call per row and chunk), and every
// `v_mfma_f32_16x16x4_f32` multiplies a 16 x 4 tile of signs (+-1.0, built from the bits) with a 4 x 16 tile
// of z.  Operands are fp32, so the products are exact and only the order of the additions differs from the
// vector kernel.  A lane (t, kg) holds sign row / token t and loads z[t][16 s + 4 kg .. + 4) of the chunk
// as one 16-byte load for s = 0..7; component jj of load s is the B operand of multiply (s, jj), whose k
// index kg therefore stands for column 16 s + 4 kg + jj.
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float sk_f32x4;
typedef sk_f32x4 f32x4_acc;
constexpr int SM_WAVES = 16;

__global__ __launch_bounds__(SM_WAVES * 64)
void sketch_rademacher_mfma_kernel(OpDesc op, OpKeys keys, const float* __restrict__ z, int B, float* __restrict__ y) {
    __shared__ float red[SM_WAVES][256];
    pick_operator(op, keys);
    z += (size_t)blockIdx.z * B * op.n;
    y += (size_t)blockIdx.z * B * op.m;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tl = lane & 15, kg = lane >> 4;
    const int row0 = blockIdx.x * 16, t0 = blockIdx.y * 16;
    const int n = op.n;
    const bool tok_ok = t0 + tl < B;
    const float* zt = z + (size_t)(tok_ok ? t0 + tl : 0) * n + kg * 4;
    const int nchunks = (n + 127) >> 7;
    sk_f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};      // two chains, so that a multiply need not wait for the one before
    for (int cc = wave; cc < nchunks; cc += SM_WAVES) {
        const int c0 = cc << 7;
        float4 zv[8];
#pragma unroll
        for (int sgrp = 0; sgrp < 8; ++sgrp) {
            const int col = c0 + sgrp * 16 + kg * 4;                   // n is a multiple of 4: a load is all in or all out
            zv[sgrp] = (tok_ok && col < n) ? *reinterpret_cast<const float4*>(zt + c0 + sgrp * 16) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        const u32x4 bits = rademacher_bits(op, (uint32_t)(row0 + tl), (uint32_t)cc);
#pragma unroll
        for (int sgrp = 0; sgrp < 8; ++sgrp) {
            // bit 16 (sgrp % 2) + 4 kg + jj of word sgrp / 2
            const uint32_t wl = bits.w[sgrp >> 1] >> (kg * 4);
            const float zc[4] = {zv[sgrp].x, zv[sgrp].y, zv[sgrp].z, zv[sgrp].w};
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int bpos = (sgrp & 1) * 16 + jj;
                const float pm = __uint_as_float(((wl << (31 - bpos)) & 0x80000000u) | 0x3F800000u);
                acc[jj & 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(pm, zc[jj], acc[jj & 1], 0, 0, 0);
            }
        }
    }
    const sk_f32x4 tot = acc[0] + acc[1];
    *reinterpret_cast<sk_f32x4*>(&red[wave][lane * 4]) = tot;
    __syncthreads();
    // element e = lane * 4 + v of a tile is (row 4 (lane / 16) + v, token lane % 16)
    if (tid < 256) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < SM_WAVES; ++w) sum += red[w][tid];
        const int row = row0 + 4 * (tid >> 6) + (tid & 3), tok = t0 + ((tid >> 2) & 15);
        if (row < op.m && tok < B) y[(size_t)tok * op.m + row] = sum * op.scale;
    }
}

// The same contraction on the bf16 matrix cores, sixteen times the rate of the fp32 ones, without
// giving up exactness of the products: a float is the sum of three bf16 numbers (its leading eight
// significant bits, the next eight, the last eight: z = h + m + l, every difference formed exactly), and a
// sign is a bf16 number, so y = S h + S m + S l with every product exact and the sums in fp32 as before.
// Splitting costs more vector instructions than the multiplies it saves unless it is shared, so here a
// workgroup owns ALL rows of Phi for one tile of 16 tokens (wave w takes the 16-row blocks w, w + 16) and a
// range of 128-column chunks: per chunk the 1024 threads split the 16 x 128 values once into three planes
// in LDS (double buffered, one barrier per chunk), and every wave multiplies its sign tiles (eight signs per
// lane and k-step packed from one byte of the row's 128 bits) with the planes by `v_mfma_f32_16x16x32_bf16`.
// The four lanes that hold one row of a sign tile would draw the same Philox block; instead lane (row, q)
// draws the block of the q-th chunk of a group of four, and each chunk fetches its words from the lane that
// drew them (`ds_bpermute`).  The column ranges of a token tile are dealt to gridDim.x workgroups (as many
// as it takes to fill the chip); their partial tiles go to a workspace and are added in a fixed order by
// sketch_partials_kernel, which also applies the scale.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 sk_bf16x8;
constexpr int SB_WAVES = 16;
constexpr int SB_ROW = 144;                            // bf16 per token row of a plane: 128 + 16 (288 bytes = 32 modulo 256: conflict-free 16-byte fragment reads, measured)
constexpr int SB_PLANE = 16 * SB_ROW;
constexpr int SB_MAX_SPLITS = 32;                      // column ranges per token tile
#ifndef SB_TARGET_WGS
#define SB_TARGET_WGS 256
#endif

template <int RBW>
__global__ __launch_bounds__(SB_WAVES * 64)
void sketch_rademacher_bf16_kernel(OpDesc op, OpKeys keys, const float* __restrict__ z, int B, float* __restrict__ partial) {
    __shared__ __attribute__((aligned(16))) uint16_t planes[2][3][SB_PLANE];
    pick_operator(op, keys);
    z += (size_t)blockIdx.z * B * op.n;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tl = lane & 15, kg = lane >> 4;
    const int n = op.n, m = op.m;
    const int t0 = blockIdx.y * 16;
    const int nchunks = (n + 127) >> 7;
    const int c_lo = (int)((long)blockIdx.x * nchunks / gridDim.x), c_hi = (int)((long)(blockIdx.x + 1) * nchunks / gridDim.x);
    // staging: thread (token st, column pair sp) of the chunk
    const int st = tid >> 6, sp = tid & 63;
    const bool st_ok = t0 + st < B;
    const float* zrow = z + (size_t)(st_ok ? t0 + st : 0) * n + 2 * sp;
    auto fetch = [&](int cc) -> float2 {
        const int col = (cc << 7) + 2 * sp;                // n is a multiple of 4: a pair is all in or all out
        return (st_ok && cc < c_hi && col < n) ? *reinterpret_cast<const float2*>(zrow + (cc << 7)) : make_float2(0.f, 0.f);
    };
    auto split_store = [&](float2 v, int buf) {
        const uint32_t a0 = __float_as_uint(v.x) & 0xFFFF0000u, b0 = __float_as_uint(v.y) & 0xFFFF0000u;
        const float ra = v.x - __uint_as_float(a0), rb = v.y - __uint_as_float(b0);
        const uint32_t a1 = __float_as_uint(ra) & 0xFFFF0000u, b1 = __float_as_uint(rb) & 0xFFFF0000u;
        const float sa = ra - __uint_as_float(a1), sb = rb - __uint_as_float(b1);
        const uint32_t a2 = __float_as_uint(sa) & 0xFFFF0000u, b2 = __float_as_uint(sb) & 0xFFFF0000u;
        uint32_t* dst = reinterpret_cast<uint32_t*>(&planes[buf][0][st * SB_ROW + 2 * sp]);
        dst[0] = (a0 >> 16) | b0;
        dst[SB_PLANE / 2] = (a1 >> 16) | b1;
        dst[SB_PLANE] = (a2 >> 16) | b2;
    };
    f32x4_acc acc[RBW];
    u32x4 drawn[RBW];                                  // Philox block of (row tl, chunk kg of the current group of four)
#pragma unroll
    for (int r = 0; r < RBW; ++r) { acc[r] = f32x4_acc{0.f, 0.f, 0.f, 0.f}; drawn[r] = u32x4{{0u, 0u, 0u, 0u}}; }
    float2 zreg = fetch(c_lo);
    for (int cc = c_lo; cc < c_hi; ++cc) {
        const int buf = (cc - c_lo) & 1;
        split_store(zreg, buf);
        zreg = fetch(cc + 1);
        __syncthreads();                               // the planes of chunk cc are complete; the other buffer is free again
        const int in_group = (cc - c_lo) & 3;
#pragma unroll
        for (int r = 0; r < RBW; ++r) {
            const int row0 = (wave + r * SB_WAVES) * 16;
            if (row0 < m) {                            // uniform over the wave
                if (in_group == 0) drawn[r] = rademacher_bits(op, (uint32_t)(row0 + tl), (uint32_t)(cc + kg));
                const int src = in_group * 16 + tl;    // the lane that drew this chunk's block for row tl
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    // columns 32 ks + 8 kg + j of the chunk: bits 8 kg + j of word ks; a set bit is -1
                    const uint32_t by = ((uint32_t)__shfl((int)drawn[r].w[ks], src) >> (kg * 8)) & 0xFFu;
                    union { uint32_t u[4]; sk_bf16x8 v; } sg;
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        sg.u[q] = 0x3F803F80u | (((by >> (2 * q)) & 1u) << 15) | (((by >> (2 * q + 1)) & 1u) << 31);
#pragma unroll
                    for (int pl = 0; pl < 3; ++pl) {
                        const sk_bf16x8 zb = *reinterpret_cast<const sk_bf16x8*>(&planes[buf][pl][tl * SB_ROW + ks * 32 + kg * 8]);
                        acc[r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sg.v, zb, acc[r], 0, 0, 0);
                    }
                }
            }
        }
    }
    // element v of a lane's tile is (row 4 (lane / 16) + v, token lane % 16); partial tiles:
    // [operator][range][token tile][16 tokens][rows, padded to 16], i.e. the layout of y
    const int rows_pad = ((m + 15) >> 4) << 4;
    float* pt = partial + ((((size_t)blockIdx.z * gridDim.x + blockIdx.x) * gridDim.y + blockIdx.y) * 16) * rows_pad;
#pragma unroll
    for (int r = 0; r < RBW; ++r) {
        const int row0 = (wave + r * SB_WAVES) * 16;
        if (row0 < m) *reinterpret_cast<f32x4_acc*>(pt + (size_t)tl * rows_pad + row0 + 4 * kg) = acc[r];
    }
}

// y[operator][token][row] = scale * sum over the column ranges of the partial tiles, in the order of the ranges
__global__ void sketch_partials_kernel(const float* __restrict__ partial, int nz, int splits, int tiles, int m, int B, float scale,
                                       float* __restrict__ y) {
    const int rows_pad = ((m + 15) >> 4) << 4;
    const long total = (long)nz * B * m;
    for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (long)gridDim.x * blockDim.x) {
        const int row = (int)(e % m);
        const int tok = (int)((e / m) % B);
        const int j = (int)(e / ((long)m * B));
        const int ty = tok >> 4, tl = tok & 15;
        // all ranges' values requested at once, added in the order of the ranges
        float v[SB_MAX_SPLITS];
#pragma unroll
        for (int q = 0; q < SB_MAX_SPLITS; ++q)
            v[q] = q < splits ? partial[((((size_t)j * splits + q) * tiles + ty) * 16 + tl) * rows_pad + row] : 0.f;
        float sum = 0.f;
#pragma unroll
        for (int q = 0; q < SB_MAX_SPLITS; ++q) sum += v[q];
        y[e] = sum * scale;
    }
}

template <int TB, bool VEC>
__global__ __launch_bounds__(SK_WAVES * 64)
void sketch_gauss_kernel(OpDesc op, OpKeys keys, const float* __restrict__ z, int B, float* __restrict__ y) {
    pick_operator(op, keys);
    z += (size_t)blockIdx.z * B * op.n;
    y += (size_t)blockIdx.z * B * op.m;
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

// The same products with the columns of a row dealt to all waves of a workgroup (one workgroup per row):
// for launches with few rows and tokens (a prompt-level sketch: one token, a few hundred rows), where one
// wave per row would leave most of the chip idle while every lane draws its hundred-odd Gaussians one after
// the other.  Wave w takes column groups w*64 + lane, + 64*nwaves, ...; the waves' sums are added in wave
// order.  The split depends on the operator's shape and the batch only, never on how many operators share
// the launch, so a multi-operator launch returns the bits of the single-operator call.
template <int TB, bool VEC>
__global__ __launch_bounds__(1024)
void sketch_gauss_split_kernel(OpDesc op, OpKeys keys, const float* __restrict__ z, int B, float* __restrict__ y) {
    __shared__ float part[16][TB];
    pick_operator(op, keys);
    z += (size_t)blockIdx.z * B * op.n;
    y += (size_t)blockIdx.z * B * op.m;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int row = blockIdx.x;
    const int t0 = blockIdx.y * TB;
    const int nt = min(TB, B - t0);
    float acc[TB];
#pragma unroll
    for (int t = 0; t < TB; ++t) acc[t] = 0.f;
    const int ngroups = (op.n + 3) >> 2;
    for (int cg = wave * 64 + lane; cg < ngroups; cg += 64 * nwaves) {
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
        if (lane == 0) part[wave][t] = s;
    }
    __syncthreads();
    if (threadIdx.x < nt) {
        float s = 0.f;
        for (int w = 0; w < nwaves; ++w) s += part[w][threadIdx.x];
        y[(size_t)(t0 + threadIdx.x) * op.m + row] = s * op.scale;
    }
}

// LDS position of transform index i: one float of padding per 32 keeps both the 16-float runs of the
// first pass and the unit-stride accesses of the later passes free of bank conflicts
__device__ __forceinline__ int wht_pos(int i) { return i + (i >> 5); }

template <int R>
__device__ __forceinline__ void wht_regs(float (&v)[1 << R]) {
#pragma unroll
    for (int lv = 0; lv < R; ++lv)
#pragma unroll
        for (int e = 0; e < (1 << R); ++e)
            if (!(e & (1 << lv))) {
                const float a = v[e], b = v[e | (1 << lv)];
                v[e] = a + b;
                v[e | (1 << lv)] = a - b;
            }
}

// butterfly levels of the index bits [sh, sh + R) on the n' = 2^nbits values in LDS
template <int R>
__device__ __forceinline__ void wht_pass(float* x, int nbits, int sh) {
    const int ngroups = 1 << (nbits - R);
    for (int g = threadIdx.x; g < ngroups; g += blockDim.x) {
        const int base = ((g >> sh) << (sh + R)) | (g & ((1 << sh) - 1));
        float v[1 << R];
#pragma unroll
        for (int e = 0; e < (1 << R); ++e) v[e] = x[wht_pos(base + (e << sh))];
        wht_regs<R>(v);
#pragma unroll
        for (int e = 0; e < (1 << R); ++e) x[wht_pos(base + (e << sh))] = v[e];
    }
}

__global__ __launch_bounds__(1024)
void sketch_srht_kernel(OpDesc op, OpKeys keys, const float* __restrict__ z, int B, float* __restrict__ y) {
    extern __shared__ float xs[];                       // 2^nbits values at their padded positions
    pick_operator(op, keys);
    z += (size_t)blockIdx.z * B * op.n;
    y += (size_t)blockIdx.z * B * op.m;
    const int npad = 1 << op.nbits;
    const int tok = blockIdx.x, tid = threadIdx.x, NT = blockDim.x;
    const float* zt = z + (size_t)tok * op.n;
    const bool vec = (op.n & 3) == 0;                   // float4 loads need 16-byte aligned rows of z
    if (op.nbits >= 4) {
        // first pass fused with the load: a thread takes 16 consecutive columns (one 16-bit run of sign
        // bits), transforms index bits 0..3 in registers and stores the run
        for (int g = tid; g < (npad >> 4); g += NT) {
            const int c0 = g << 4;
            float v[16];
            if (c0 < op.n) {
                const u32x4 b = srht_sign_bits(op, (uint32_t)c0 >> 7);
                const uint32_t bits = b.w[(c0 & 127) >> 5] >> (c0 & 31);
                if (vec && c0 + 16 <= op.n) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float4 t = *reinterpret_cast<const float4*>(zt + c0 + 4 * q);
                        v[4 * q] = t.x; v[4 * q + 1] = t.y; v[4 * q + 2] = t.z; v[4 * q + 3] = t.w;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 16; ++e) v[e] = c0 + e < op.n ? zt[c0 + e] : 0.f;
                }
#pragma unroll
                for (int e = 0; e < 16; ++e) v[e] = __uint_as_float(__float_as_uint(v[e]) ^ (((bits >> e) & 1u) << 31));
                wht_regs<4>(v);
            } else {
#pragma unroll
                for (int e = 0; e < 16; ++e) v[e] = 0.f;
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) xs[wht_pos(c0 + e)] = v[e];
        }
    } else {
        for (int c = tid; c < npad; c += NT) {
            float v = 0.f;
            if (c < op.n) {
                const u32x4 b = srht_sign_bits(op, 0u);
                v = __uint_as_float(__float_as_uint(zt[c]) ^ (((b.w[0] >> c) & 1u) << 31));
            }
            xs[wht_pos(c)] = v;
        }
    }
    __syncthreads();
    int sh = op.nbits >= 4 ? 4 : 0;
    for (; sh + 4 <= op.nbits; sh += 4) { wht_pass<4>(xs, op.nbits, sh); __syncthreads(); }
    const int rest = op.nbits - sh;
    if (rest == 3) wht_pass<3>(xs, op.nbits, sh);
    else if (rest == 2) wht_pass<2>(xs, op.nbits, sh);
    else if (rest == 1) wht_pass<1>(xs, op.nbits, sh);
    __syncthreads();
    const SrhtRows key = srht_rows_key(op);
    for (int i = tid; i < op.m; i += NT) y[(size_t)tok * op.m + i] = xs[wht_pos((int)srht_row(key, (uint32_t)i))] * op.scale;
}

constexpr int SRHT_MAX_BITS = 15;                       // 128 KB of LDS for the values

bool sketch_srht_supported(const OpDesc& op) { return op.nbits <= SRHT_MAX_BITS; }

// ops[0..n_ops): operators of one ensemble and shape; z [n_ops][B][n], y [n_ops][B][m].
hipError_t launch_sketch_multi(const OpDesc* ops, int n_ops, const float* z, int B, float* y, hipStream_t s,
                               void* scratch, size_t scratch_bytes) {
    if (B <= 0 || n_ops <= 0) return hipSuccess;
    const OpDesc& op = ops[0];
    if (op.ens == 2 && !sketch_srht_supported(op)) return hipErrorInvalidValue;
    for (int j0 = 0; j0 < n_ops; j0 += SK_MAX_OPS) {
        const int nz = n_ops - j0 < SK_MAX_OPS ? n_ops - j0 : SK_MAX_OPS;
        OpKeys keys;
        for (int j = 0; j < SK_MAX_OPS; ++j) {
            const OpDesc& o = ops[j0 + (j < nz ? j : 0)];
            keys.k0[j] = o.k0; keys.k1[j] = o.k1; keys.stream[j] = o.stream;
        }
        const float* zj = z + (size_t)j0 * B * op.n;
        float* yj = y + (size_t)j0 * B * op.m;
        if (op.ens == 2) {
            const int npad = 1 << op.nbits;
            const size_t bytes = (size_t)(npad + (npad >> 5) + 4) * 4;
            static size_t allowed = 0;
            if (bytes > allowed) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(sketch_srht_kernel),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
                if (e != hipSuccess) return e;
                allowed = bytes;
            }
            int nthreads = npad / 16;
            nthreads = nthreads < 64 ? 64 : (nthreads > 1024 ? 1024 : nthreads);
            hipLaunchKernelGGL(sketch_srht_kernel, dim3(B, 1, nz), dim3(nthreads), bytes, s, op, keys, zj, B, yj);
        } else if (op.ens == 1) {
            const int tgroups = (B + 7) / 8;
            const long mfma_wgs = (long)((op.m + 15) / 16) * ((B + 15) / 16) * nz;
            const int tiles = (B + 15) / 16, rows_pad = ((op.m + 15) / 16) * 16, nchunks = (op.n + 127) / 128;
            int splits = (SB_TARGET_WGS + nz * tiles - 1) / (nz * tiles);       // column ranges per token tile: fill the chip
            splits = splits < 1 ? 1 : (splits > SB_MAX_SPLITS ? SB_MAX_SPLITS : splits);
            if (splits > nchunks) splits = nchunks;
            const size_t part_bytes = (size_t)nz * splits * tiles * rows_pad * 16 * sizeof(float);
            if ((op.n & 3) == 0 && mfma_wgs >= 128 && op.m <= 512 && scratch && part_bytes <= scratch_bytes) {
                // enough 16 x 16 tiles to fill the chip (several operators per launch): bf16 matrix cores on the
                // three-way split of z, partial tiles per column range in the workspace, then their sum
                float* part = static_cast<float*>(scratch);
                const dim3 grid(splits, tiles, nz);
                if (op.m <= 256) hipLaunchKernelGGL((sketch_rademacher_bf16_kernel<1>), grid, dim3(SB_WAVES * 64), 0, s, op, keys, zj, B, part);
                else hipLaunchKernelGGL((sketch_rademacher_bf16_kernel<2>), grid, dim3(SB_WAVES * 64), 0, s, op, keys, zj, B, part);
                const long total = (long)nz * B * op.m;
                const int rgrid = (int)((total + 255) / 256 < 1024 ? (total + 255) / 256 : 1024);
                hipLaunchKernelGGL(sketch_partials_kernel, dim3(rgrid), dim3(256), 0, s, part, nz, splits, tiles, op.m, B, op.scale, yj);
            } else if ((op.n & 3) == 0 && mfma_wgs >= 128) {
                // the same without a workspace (or more than 512 rows): fp32 matrix cores
                hipLaunchKernelGGL(sketch_rademacher_mfma_kernel, dim3((op.m + 15) / 16, (B + 15) / 16, nz), dim3(SM_WAVES * 64), 0, s,
                                   op, keys, zj, B, yj);
            } else if ((long)((op.m + 3) / 4) * tgroups * nz >= 256) {
                hipLaunchKernelGGL((sketch_rademacher_kernel<4, 8>), dim3((op.m + 3) / 4, tgroups, nz), dim3(SR_WAVES * 64), 0, s, op, keys, zj, B, yj);
            } else {
                hipLaunchKernelGGL((sketch_rademacher_kernel<2, 8>), dim3((op.m + 1) / 2, tgroups, nz), dim3(SR_WAVES * 64), 0, s, op, keys, zj, B, yj);
            }
        } else {
            const bool vec = (op.n & 3) == 0;   // float4 loads need 16-byte aligned rows of z
            // few rows x token groups per operator: deal each row's columns to several waves
            const long waves = (long)op.m * ((B + SK_TB - 1) / SK_TB);
            const int useful = (((op.n + 3) >> 2) + 63) / 64;          // waves that get at least one column group
            int split = 1;
            while (split < 16 && waves * split < 2048 && split * 2 <= useful) split *= 2;
            if (split > 1) {
                dim3 sgrid(op.m, (B + SK_TB - 1) / SK_TB, nz);
                if (vec) hipLaunchKernelGGL((sketch_gauss_split_kernel<SK_TB, true>), sgrid, dim3(split * 64), 0, s, op, keys, zj, B, yj);
                else hipLaunchKernelGGL((sketch_gauss_split_kernel<SK_TB, false>), sgrid, dim3(split * 64), 0, s, op, keys, zj, B, yj);
                continue;
            }
            dim3 grid((op.m + SK_WAVES - 1) / SK_WAVES, (B + SK_TB - 1) / SK_TB, nz);
            if (vec) hipLaunchKernelGGL((sketch_gauss_kernel<SK_TB, true>), grid, dim3(SK_WAVES * 64), 0, s, op, keys, zj, B, yj);
            else hipLaunchKernelGGL((sketch_gauss_kernel<SK_TB, false>), grid, dim3(SK_WAVES * 64), 0, s, op, keys, zj, B, yj);
        }
    }
    return hipGetLastError();
}

hipError_t launch_sketch(const OpDesc& op, const float* z, int B, float* y, hipStream_t s) {
    return launch_sketch_multi(&op, 1, z, B, y, s, nullptr, 0);
}

}  // namespace csk
