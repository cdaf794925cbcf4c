// Block-sparse gated FFN as two gathered matrix products on the matrix cores, for
// many rows per call: one shared support (task-conditioned prefill, paper Sec. 4)
// or per-row supports over their union with a mask (token-adaptive batches, Sec. 5).
// Here the path really is a dense contraction over the gathered blocks:
//   H   = silu(X Wg_S^T) * (X Wu_S^T)      [T x |S|*64]   (K = d)
//   out = H Wd_S                           [T x d]        (K = |S|*64)
// Both products have K-contiguous operands (X and the weight rows for the first; H
// and the [d][64] block slices of Wd for the second), so every tile is filled with
// 16-byte loads.  Workgroup tile 128 x 128 (first product: 64 gate + 64 up columns
// of one block), K step 64, four waves of 64 x 64, mfma_f32_32x32x16_bf16, fp32
// accumulation, LDS double buffered with the next tile's global loads in flight
// during the multiplies.  LDS rows are 128 bytes; the eight 16-byte chunks of a row
// are stored XOR-swizzled by the row index so that fragment reads are conflict free.
#include "kernels.hpp"
#include "common.hpp"
#include <type_traits>

namespace csk {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

constexpr int GM_BM = 128, GM_BN = 128, GM_BK = 64, GM_THREADS = 256;

struct GemmArgs {
    const uint16_t *Wg, *Wu, *Wd;
    const uint16_t* x;
    uint16_t* hid;            // [T][nb*64]
    uint16_t* out;            // [T][d]
    float* partial;           // [splits][T][d] fp32, split-K only
    const int32_t* blocks;    // block index per slot of the gathered list
    const int32_t* nblocks;   // device scalar: number of slots in use
    const uint32_t* mask;     // [G][mask_words] token bitsets, or nullptr (every row uses every listed block)
    int mask_words;
    int T, d, G, nb_max;      // nb_max: row length of hid / 64
};

// LDS serves a 16-byte read per lane sixteen lanes at a time: lanes 0-7 with 24-31 and 8-15 with 16-23 of each half
// of the wave, and the sixteen have to fall into different 16-byte columns of the 256-byte bank row (measured: a
// fragment read takes 1.6 times as long otherwise).  A fragment read has lane = row % 32 + 32 * (chunk % 2), so the
// swizzle takes bit 4 of the row along with the low bits.
__device__ __forceinline__ int swz_of(int row) { return ((row >> 1) & 3) | (((row >> 4) & 1) << 2); }
__device__ __forceinline__ int swz(int row, int chunk) { return (row << 3) + (chunk ^ swz_of(row)); }

// rows of a [32 x 32] accumulator: register j of lane L is (row 8*(j/4) + 4*(L/32) + j%4, column L%32)
__device__ __forceinline__ int acc_row(int j, int lane) { return 8 * (j >> 2) + 4 * (lane >> 5) + (j & 3); }

// MODE 0: gate/up product with the activation epilogue; MODE 1: down product.
// BM: rows per workgroup tile (128, or 64 for short batches).  SPLITK (MODE 1 only): the K range is
// divided over gridDim.z workgroups that write fp32 partial tiles, summed by ffn_splitk_reduce_kernel.
template <int MODE, int BM, bool SPLITK>
__global__ __launch_bounds__(GM_THREADS)
void ffn_gemm_kernel(GemmArgs a) {
    constexpr int MI = BM / 64;                       // 32-row tiles per wave
    constexpr int ACH = BM / 32;                      // 16-byte chunks of A per thread and tile
    __shared__ bf16x8_t As[2][BM * 8];
    __shared__ bf16x8_t Bs[2][GM_BN * 8];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int nb = *a.nblocks;
    const int bm = blockIdx.y * BM;
    const int d = a.d, T = a.T;
    const int ldh = a.nb_max * 64;
    int kt0 = 0, kt1, g0 = 0, bn = 0;
    if (MODE == 0) {
        if ((int)blockIdx.x >= nb) return;
        g0 = a.blocks[blockIdx.x];
        kt1 = d / GM_BK;
    } else {
        bn = blockIdx.x * GM_BN;
        kt1 = nb;
        if (SPLITK) {
            const int per = (nb + (int)gridDim.z - 1) / (int)gridDim.z;
            kt0 = blockIdx.z * per;
            kt1 = min(nb, kt0 + per);
        }
    }
    const int ktiles = kt1 > kt0 ? kt1 - kt0 : 0;
    // global -> register staging: 16-byte chunks of A and of B per thread and tile.  Two tiles are
    // kept in flight (register sets 0 and 1) besides the one being multiplied out of LDS.
    bf16x8_t ra[2][ACH], rb[2][4];
    auto fetch = [&](int set, int kt) {
        kt += kt0;
        const bf16x8_t zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < ACH; ++i) {
            const int id = tid + GM_THREADS * i, row = id >> 3, c = id & 7;
            if (MODE == 0)
                ra[set][i] = (bm + row < T) ? *reinterpret_cast<const bf16x8_t*>(a.x + (size_t)(bm + row) * d + kt * GM_BK + c * 8) : zero;
            else
                ra[set][i] = (bm + row < T) ? *reinterpret_cast<const bf16x8_t*>(a.hid + (size_t)(bm + row) * ldh + kt * 64 + c * 8) : zero;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = tid + GM_THREADS * i, row = id >> 3, c = id & 7;
            if (MODE == 0) {
                const uint16_t* w = row < 64 ? a.Wg + ((size_t)g0 * 64 + row) * d : a.Wu + ((size_t)g0 * 64 + row - 64) * d;
                rb[set][i] = *reinterpret_cast<const bf16x8_t*>(w + kt * GM_BK + c * 8);
            } else {
                const int g = a.blocks[kt];
                rb[set][i] = (bn + row < d) ? *reinterpret_cast<const bf16x8_t*>(a.Wd + ((size_t)g * d + bn + row) * 64 + c * 8) : zero;
            }
        }
    };
    auto stash = [&](int set, int buf) {
#pragma unroll
        for (int i = 0; i < ACH; ++i) {
            const int id = tid + GM_THREADS * i, row = id >> 3, c = id & 7;
            As[buf][swz(row, c)] = ra[set][i];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = tid + GM_THREADS * i, row = id >> 3, c = id & 7;
            Bs[buf][swz(row, c)] = rb[set][i];
        }
    };
    f32x16_t acc[MI][2];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int lr = lane & 31, lk = lane >> 5;
    // tile t >= 1 travels in register set (t - 1) & 1
    if (ktiles > 0) { fetch(0, 0); stash(0, 0); }
    if (ktiles > 1) fetch(0, 1);
    if (ktiles > 2) fetch(1, 2);
    __syncthreads();
    for (int kt = 0; kt < ktiles; kt += 2) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int t = kt + half;
            if (t >= ktiles) break;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                bf16x8_t fa[MI], fb[2];
#pragma unroll
                for (int i = 0; i < MI; ++i) fa[i] = As[half][swz(wm * (BM / 2) + i * 32 + lr, kk * 2 + lk)];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    // first product: column tile j = 0 is gate, j = 1 the matching up channels
                    const int row = (MODE == 0) ? (j * 64 + wn * 32 + lr) : (wn * 64 + j * 32 + lr);
                    fb[j] = Bs[half][swz(row, kk * 2 + lk)];
                }
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
            if (t + 1 < ktiles) {
                stash(half, half ^ 1);                 // tile t+1 sits in set t & 1 = half
                if (t + 3 < ktiles) fetch(half, t + 3);
            }
            __syncthreads();
        }
    }
    // epilogue
    if (MODE == 0) {
        const int n = wn * 32 + lr;                  // channel inside the block
        const uint32_t* mrow = a.mask ? a.mask + (size_t)g0 * a.mask_words : nullptr;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = bm + wm * (BM / 2) + i * 32 + acc_row(e, lane);
                if (m < T) {
                    const float gt = acc[i][0][e], up = acc[i][1][e];
                    float hv = gt / (1.0f + __expf(-gt)) * up;
                    if (mrow && !((mrow[m >> 5] >> (m & 31)) & 1u)) hv = 0.f;
                    a.hid[(size_t)m * ldh + blockIdx.x * 64 + n] = f32_to_bf16(hv);
                }
            }
    } else {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int m = bm + wm * (BM / 2) + i * 32 + acc_row(e, lane);
                    const int n = bn + wn * 64 + j * 32 + lr;
                    if (m < T && n < d) {
                        if (SPLITK) a.partial[((size_t)blockIdx.z * T + m) * d + n] = acc[i][j][e];
                        else a.out[(size_t)m * d + n] = f32_to_bf16(acc[i][j][e]);
                    }
                }
    }
}

// ---------------------------------------------------------------------------
// Wide tiles for long batches (T >= 512).  With 128 x 128 tiles the multiplies wait for the
// compute unit's load path (64 bytes per cycle) and for LDS (every operand byte is written once
// and read back twice), so here one workgroup owns a 256 x 256 tile: four waves of 128 x 128
// (256 accumulator registers per lane, one wave per SIMD), K step 32, four LDS stages of 32 KB.
// The operands go from global memory straight into LDS (global_load_lds_dwordx4: lane p of a
// wave fills bytes 16p .. 16p+15 of a 1 KB run, i.e. 16 rows of 64 bytes), which needs no staging
// registers; the XOR swizzle that keeps the fragment reads conflict free is applied on the global
// side, by choosing which 16-byte chunk of its row a lane fetches.  Tiles travel in pairs (a
// 64-column step) through four stages; a stage is refilled with the tile two pairs ahead as soon as
// every wave has read it for the last time (two barriers per pair), its loads spread one per four
// multiplies over the next two k-steps.  Fragment reads for the next k-step are spread between the
// multiplies of the current one.
// ---------------------------------------------------------------------------
constexpr int GW_BM = 256, GW_BN = 256, GW_BK = 32;
#ifndef CS_GW_MIN_WGS
#define CS_GW_MIN_WGS 150
#endif
constexpr int GW_MIN_WGS = CS_GW_MIN_WGS;              // fewer wide workgroups than this: use the 128 x 128 tiles
constexpr int GW_STAGE = (GW_BM + GW_BN) * 4;          // 16-byte entries per stage
constexpr int GW_MAX_BLOCKS = 4096;                    // longest gathered list the down product keeps in LDS

// rows of 64 bytes: four rows fill a bank row, and of the rows read together (see swz) those that share row % 4
// differ in bits 2 and 4
__device__ __forceinline__ int swz4_of(int row) { return ((row >> 2) & 1) | (((row >> 4) & 1) << 1); }
__device__ __forceinline__ int swz4(int row, int chunk) { return (row << 2) + (chunk ^ swz4_of(row)); }

// One wave copies 1 KB from global memory into LDS without passing through registers: lane p
// supplies the address of its 16 bytes, which land at lds_wave_base + 16 p.  The instruction takes
// the LDS base from M0, which nothing else in these kernels uses.  It is counted by vmcnt like any
// other load; the compiler does not see it, so the kernel waits for it explicitly.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load_to_lds_16(const void* gptr, const void* lds_wave_base) {
    const unsigned l = __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)((const __attribute__((address_space(3))) void*)lds_wave_base));
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(l) : "memory", "m0");
}
#pragma clang diagnostic pop

template <int MODE>
__global__ __launch_bounds__(GM_THREADS) __attribute__((amdgpu_waves_per_eu(1, 1)))
void ffn_gemm_wide_kernel(GemmArgs a) {
    __shared__ bf16x8_t S[4][GW_STAGE];
    __shared__ int32_t blk_lds[MODE == 1 ? GW_MAX_BLOCKS : 1];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    // the block list is read through the scalar cache (constant address space), never by a vector
    // load, whose in-order completion would drain the tiles in flight
    const __attribute__((address_space(4))) int32_t* blocks = (const __attribute__((address_space(4))) int32_t*)a.blocks;
    const int nb = *a.nblocks;
    const int bm = blockIdx.y * GW_BM;
    const int d = a.d, T = a.T;
    const int ldh = a.nb_max * 64;
    int ktiles, bn = 0, g2[2] = {0, 0};
    if (MODE == 0) {
        if ((int)blockIdx.x * 2 >= nb) return;
        g2[0] = blocks[blockIdx.x * 2];
        g2[1] = blocks[min((int)blockIdx.x * 2 + 1, nb - 1)];
        ktiles = d / GW_BK;
    } else {
        bn = blockIdx.x * GW_BN;
        ktiles = nb * 2;                               // always even, like d / 32
        for (int i = tid; i < nb; i += GM_THREADS) blk_lds[i] = a.blocks[i];   // visible after the first barrier
    }
    // Per lane and load instruction: the row it fetches and the chunk of that row.  Instruction u of
    // wave w covers tile rows 16 (4u + w) .. +15; lane p takes row p / 4, LDS slot p % 4.
    const uint16_t* pa[4];
    const uint16_t* pb[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int r = (u * 4 + wave) * 16 + (lane >> 2);
        const int chunk = (lane & 3) ^ swz4_of(r);
        const int m = min(bm + r, T - 1);              // rows past T repeat the last row; never stored
        pa[u] = (MODE == 0 ? a.x + (size_t)m * d : a.hid + (size_t)m * ldh) + chunk * 8;
        if (MODE == 0) {
            const int g = g2[r >> 7], c = r & 127;
            pb[u] = (c < 64 ? a.Wg + ((size_t)g * 64 + c) * d : a.Wu + ((size_t)g * 64 + c - 64) * d) + chunk * 8;
        } else {
            pb[u] = a.Wd + (size_t)min(bn + r, d - 1) * 64 + chunk * 8;
        }
    }
    // Tiles travel in pairs (a 64-column step, one block of the down product): pair q lives in stages
    // 2 (q & 1) (its first tile) and 2 (q & 1) + 1 (its second); a pair past the last one repeats the last
    // one and is never multiplied.  A stage takes 8 loads per wave (4 parts of A rows, 4 parts of B rows);
    // they are issued one per four multiplies, spread over two k-steps, because the compute unit's load
    // path takes 16 cycles per instruction and wave: sixteen of them inside one k-step (32 KB for the
    // workgroup against 512 cycles of multiplies) made that k-step three times as long as the others.
    // Inside the loop the block id of the down product comes from a copy of the list in LDS: LDS
    // reads complete in order, so waiting for it does not drain the fragment reads in flight the
    // way a scalar load's wait would (and a vector load's wait would drain the tiles in flight).
    const int plast = ktiles / 2 - 1;
    struct Refill { const bf16x8_t* St; size_t ao, bo; };
    auto refill_of = [&](int q, int second, uint32_t g) {
        Refill r;
        r.St = S[2 * (q & 1) + second];
        r.ao = (size_t)min(q, plast) * (2 * GW_BK) + second * GW_BK;
        r.bo = MODE == 0 ? r.ao : (size_t)g * d * 64 + second * GW_BK;
        return r;
    };
    // load i (0..7) of a stage: part i / 2 of the A rows (even i) or of the B rows (odd i)
    auto issue_one = [&](const Refill& r, int i) {
        const int u = i >> 1;
        if ((i & 1) == 0) load_to_lds_16(pa[u] + r.ao, r.St + (u * 4 + wave) * 64);
        else load_to_lds_16(pb[u] + r.bo, r.St + GW_BM * 4 + (u * 4 + wave) * 64);
    };
    auto block_of = [&](int q, bool from_lds) -> uint32_t {
        if (MODE != 1) return 0u;
        return from_lds ? (uint32_t)blk_lds[min(q, plast)] : (uint32_t)blocks[min(q, plast)];
    };
    f32x16_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    const int lr = lane & 31, lk = lane >> 5;
    bf16x8_t fa[2][4], fb[2][4];
    // Fragment reads of k-step kk of tile t, in four parts of two: the B fragments first (every
    // row of multiplies needs all four of them), then the A fragments in the order of use.
    auto frag_pair = [&](int set, int t, int kk, int i) {
        const bf16x8_t* St = S[t & 3];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int f = (i & 1) * 2 + h;
            // first product: the wave's 128 columns are one block, gate channels then up channels
            if (i < 2) fb[set][f] = St[GW_BM * 4 + swz4(wn * 128 + f * 32 + lr, kk * 2 + lk)];
            else fa[set][f] = St[swz4(wm * 128 + f * 32 + lr, kk * 2 + lk)];
        }
    };
    auto frags = [&](int set, int t, int kk) {
#pragma unroll
        for (int i = 0; i < 4; ++i) frag_pair(set, t, kk, i);
    };
    auto multiply_row = [&](int set, int i) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
    };
    // The order below is pinned with scheduling barriers: left alone, the compiler sinks every
    // fragment read next to its first use, which exposes the LDS latency four times per tile.
    // A pair is four k-steps of 16 multiplies; k-step s multiplies fragment set s & 1 while the next
    // k-step's fragments are read into the other set.  Two workgroup barriers per pair: after the first
    // k-step every wave has read the pair's first stage for the last time, after the third the second
    // stage.  A freed stage is refilled with the tile two pairs ahead over the next two k-steps.  In issue
    // order the loads of a wave are: first tile of pair q+2 (k-steps 2, 3 of pair q), second tile of pair
    // q+2 (k-step 4 of pair q, k-step 1 of pair q+1), first tile of pair q+3, ...  A barrier that must see
    // a tile landed (the second tile of pair q at the first barrier, the first tile of pair q+1 at the
    // second) therefore has exactly two younger stages in flight: s_waitcnt vmcnt(16), with lgkmcnt(0)
    // for the wave's own fragment reads of the stage that is about to be refilled.
    if (ktiles > 0) {
        {
            const uint32_t g0 = block_of(0, false), g1 = block_of(1, false);
            const Refill r00 = refill_of(0, 0, g0), r01 = refill_of(0, 1, g0), r10 = refill_of(1, 0, g1), r11 = refill_of(1, 1, g1);
#pragma unroll
            for (int i = 0; i < 8; ++i) issue_one(r00, i);
#pragma unroll
            for (int i = 0; i < 8; ++i) issue_one(r01, i);
#pragma unroll
            for (int i = 0; i < 8; ++i) issue_one(r10, i);
#pragma unroll
            for (int i = 0; i < 8; ++i) issue_one(r11, i);
        }
        __builtin_amdgcn_s_waitcnt(0x4070);            // pair 0 has landed (pair 1 still in flight)
        __syncthreads();
        frags(0, 0, 0);
        // one k-step: the 16 multiplies of fragment set `set`, with the reads of the next k-step's
        // fragments (two per four multiplies) and four loads of a refill (one per four multiplies)
        // spread between them
        auto kstep = [&](int set, int tn, int kkn, const Refill& r, int half, bool loads) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                frag_pair(set ^ 1, tn, kkn, i);
                multiply_row(set, i);
                if (loads) issue_one(r, 4 * half + i);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        uint32_t g_prev = block_of(1, false);          // block of pair q + 1
        for (int q = 0; q <= plast; ++q) {
            const int t = 2 * q;
            const uint32_t g_next = block_of(q + 2, true);
            const Refill rb_prev = refill_of(q + 1, 1, g_prev);     // second tile of pair q + 1, half issued already
            kstep(0, t, 1, rb_prev, 1, q > 0);
            __builtin_amdgcn_s_waitcnt(0x4070);        // second tile of pair q landed; own reads of the first stage done
            __syncthreads();
            const Refill ra = refill_of(q + 2, 0, g_next);
            kstep(1, t + 1, 0, ra, 0, true);
            kstep(0, t + 1, 1, ra, 1, true);
            __builtin_amdgcn_s_waitcnt(0x4070);        // first tile of pair q + 1 landed; own reads of the second stage done
            __syncthreads();
            const Refill rb = refill_of(q + 2, 1, g_next);
            kstep(1, t + 2, 0, rb, 0, true);
            g_prev = g_next;
        }
        __builtin_amdgcn_s_waitcnt(0x0070);            // surplus fetches land before the LDS is released
    }
    if (MODE == 0) {
        const int slot = blockIdx.x * 2 + wn;
        if (slot >= nb) return;
        const uint32_t* mrow = a.mask ? a.mask + (size_t)g2[wn] * a.mask_words : nullptr;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int m = bm + wm * 128 + i * 32 + acc_row(e, lane);
                    if (m < T) {
                        const float gt = acc[i][j][e], up = acc[i][j + 2][e];
                        float hv = gt / (1.0f + __expf(-gt)) * up;
                        if (mrow && !((mrow[m >> 5] >> (m & 31)) & 1u)) hv = 0.f;
                        a.hid[(size_t)m * ldh + slot * 64 + j * 32 + lr] = f32_to_bf16(hv);
                    }
                }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int m = bm + wm * 128 + i * 32 + acc_row(e, lane);
                    const int n = bn + wn * 128 + j * 32 + lr;
                    if (m < T && n < d) a.out[(size_t)m * d + n] = f32_to_bf16(acc[i][j][e]);
                }
    }
}

// out = sum over the K splits of the fp32 partial tiles, in a fixed order
__global__ void ffn_splitk_reduce_kernel(const float* __restrict__ partial, int splits, size_t n, uint16_t* __restrict__ out) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float s = 0.f;
    for (int k = 0; k < splits; ++k) s += partial[(size_t)k * n + i];
    out[i] = f32_to_bf16(s);
}

// Gathered block list for per-row supports: token bitsets per block and the ordered
// list of blocks used by at least one row.  One workgroup.
__global__ __launch_bounds__(1024)
void ffn_union_kernel(const int32_t* __restrict__ support, int T, int k, int G, int mask_words,
                      uint32_t* __restrict__ mask, int32_t* __restrict__ blocks, int32_t* __restrict__ nblocks) {
    __shared__ int wcount[16];
    __shared__ int base;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < G * mask_words; i += 1024) mask[i] = 0u;
    if (tid == 0) base = 0;
    __syncthreads();
    __threadfence_block();
    for (int i = tid; i < T * k; i += 1024) {
        const int g = support[i], t = i / k;
        if (g >= 0 && g < G) atomicOr(&mask[(size_t)g * mask_words + (t >> 5)], 1u << (t & 31));
    }
    __syncthreads();
    for (int g0 = 0; g0 < G; g0 += 1024) {
        const int g = g0 + tid;
        bool used = false;
        if (g < G)
            for (int w = 0; w < mask_words; ++w) used |= mask[(size_t)g * mask_words + w] != 0u;
        const unsigned long long bal = __ballot(used);
        if (lane == 0) wcount[wave] = __popcll(bal);
        __syncthreads();
        int off = base;
        for (int w = 0; w < wave; ++w) off += wcount[w];
        if (used) blocks[off + __popcll(bal & ((1ull << lane) - 1ull))] = g;
        __syncthreads();
        if (tid == 0) { int tot = 0; for (int w = 0; w < 16; ++w) tot += wcount[w]; base += tot; }
        __syncthreads();
    }
    if (tid == 0) *nblocks = base;
}

// Shared support: copy the list (dropping out-of-range entries) and its length.
__global__ void ffn_shared_list_kernel(const int32_t* __restrict__ support, int k, int G,
                                       int32_t* __restrict__ blocks, int32_t* __restrict__ nblocks) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        int n = 0;
        for (int i = 0; i < k; ++i) { const int g = support[i]; if (g >= 0 && g < G) blocks[n++] = g; }
        *nblocks = n;
    }
}

bool ffn_gemm_ok(const FfnArgs& a) {
    return a.dtype == 1 && a.b == 64 && (a.d % 64) == 0 && a.T > 16;
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// short batches: 64-row tiles and a split of the down product's K range over 8 workgroups
static bool gemm_short(const FfnArgs& a) { return a.T <= 64; }
constexpr int GM_SPLITS = 8;

size_t ffn_gemm_scratch_bytes(const FfnArgs& a) {
    const int nb_max = a.shared ? a.k : (a.G < a.T * a.k ? a.G : a.T * a.k);
    const int mask_words = (a.T + 31) / 32;
    return align256((size_t)a.T * nb_max * 64 * 2) + align256((size_t)a.G * 4 + 4) +
           (a.shared ? 0 : align256((size_t)a.G * mask_words * 4)) +
           (gemm_short(a) ? align256((size_t)GM_SPLITS * a.T * a.d * 4) : 0) + 256;
}

hipError_t launch_ffn_gemm(const FfnArgs& a, hipStream_t s) {
    const int nb_max = a.shared ? a.k : (a.G < a.T * a.k ? a.G : a.T * a.k);
    const int mask_words = (a.T + 31) / 32;
    char* p = static_cast<char*>(a.scratch);
    GemmArgs g;
    g.hid = reinterpret_cast<uint16_t*>(p); p += align256((size_t)a.T * nb_max * 64 * 2);
    int32_t* blocks = reinterpret_cast<int32_t*>(p);
    int32_t* nblocks = blocks + a.G;
    p += align256((size_t)a.G * 4 + 4);
    uint32_t* mask = nullptr;
    if (!a.shared) { mask = reinterpret_cast<uint32_t*>(p); p += align256((size_t)a.G * mask_words * 4); }
    g.partial = reinterpret_cast<float*>(p);
    g.Wg = (const uint16_t*)a.Wg; g.Wu = (const uint16_t*)a.Wu; g.Wd = (const uint16_t*)a.Wd;
    g.x = (const uint16_t*)a.x; g.out = (uint16_t*)a.out;
    g.blocks = blocks; g.nblocks = nblocks; g.mask = mask; g.mask_words = mask_words;
    g.T = a.T; g.d = a.d; g.G = a.G; g.nb_max = nb_max;
    if (a.shared) hipLaunchKernelGGL(ffn_shared_list_kernel, dim3(1), dim3(64), 0, s, a.support, a.k, a.G, blocks, nblocks);
    else hipLaunchKernelGGL(ffn_union_kernel, dim3(1), dim3(1024), 0, s, a.support, a.T, a.k, a.G, mask_words, mask, blocks, nblocks);
    const int nt = (a.d + GM_BN - 1) / GM_BN;
    if (gemm_short(a)) {
        hipLaunchKernelGGL((ffn_gemm_kernel<0, 64, false>), dim3(nb_max, 1), dim3(GM_THREADS), 0, s, g);
        hipLaunchKernelGGL((ffn_gemm_kernel<1, 64, true>), dim3(nt, 1, GM_SPLITS), dim3(GM_THREADS), 0, s, g);
        const size_t n = (size_t)a.T * a.d;
        hipLaunchKernelGGL(ffn_splitk_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                           g.partial, GM_SPLITS, n, g.out);
    } else if (a.T >= 512 && (a.d % GW_BK) == 0 && nb_max <= GW_MAX_BLOCKS) {
        // per product: the wide tiles only when they give the chip enough workgroups, else the 128 x 128 ones
        const int mt = (a.T + GW_BM - 1) / GW_BM, mtn = (a.T + GM_BM - 1) / GM_BM;
        const int w0 = (nb_max + 1) / 2, w1 = (a.d + GW_BN - 1) / GW_BN;
        if (w0 * mt >= GW_MIN_WGS) hipLaunchKernelGGL((ffn_gemm_wide_kernel<0>), dim3(w0, mt), dim3(GM_THREADS), 0, s, g);
        else hipLaunchKernelGGL((ffn_gemm_kernel<0, GM_BM, false>), dim3(nb_max, mtn), dim3(GM_THREADS), 0, s, g);
        if (w1 * mt >= GW_MIN_WGS) hipLaunchKernelGGL((ffn_gemm_wide_kernel<1>), dim3(w1, mt), dim3(GM_THREADS), 0, s, g);
        else hipLaunchKernelGGL((ffn_gemm_kernel<1, GM_BM, false>), dim3(nt, mtn), dim3(GM_THREADS), 0, s, g);
    } else {
        const int mt = (a.T + GM_BM - 1) / GM_BM;
        hipLaunchKernelGGL((ffn_gemm_kernel<0, GM_BM, false>), dim3(nb_max, mt), dim3(GM_THREADS), 0, s, g);
        hipLaunchKernelGGL((ffn_gemm_kernel<1, GM_BM, false>), dim3(nt, mt), dim3(GM_THREADS), 0, s, g);
    }
    return hipGetLastError();
}

}  // namespace csk
