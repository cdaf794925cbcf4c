// Block-sparse gated feed-forward layer for token-adaptive batches of 17 to 64 rows (paper Sec. 5: every
// token has its own support; Sec. 7: the units are blocks of contiguous channels), bf16.
//
// Like the path for up to 16 rows, the layer is bound by the memory system: every block listed by at
// least one token has to be read once, and 64 rows per weight byte are far from filling the matrix cores.
// What changes against the 16-row kernels is where the token rows live.  Sixteen rows fit into the
// registers of the waves that split the reduction index; sixty-four do not (they would take the whole
// register file of a compute unit).  So here
//   gate/up : the channels of all listed blocks form one range cut into gridDim.x equal pieces, so every
//             workgroup streams the same number of bytes.  A workgroup takes its piece in passes of a
//             few tiles of 8 channels (8 gate rows + 8 up rows each); its waves split the reduction index
//             (within a chunk of 512 columns wave w owns columns 64 w .. 64 w + 63, so the workgroup
//             reads 1 KB of consecutive addresses of every weight row per chunk), weights go
//             global -> registers -> matrix core, one chunk ahead; the token rows are staged chunk by
//             chunk through LDS, shared by the waves, and come from L2 (every workgroup reads the same
//             rows).  Accumulators stay in registers over the whole reduction index and the waves'
//             partial tiles are summed through LDS once per pass.
//   down    : as for 16 rows (a workgroup owns 16 output columns, waves split the blocks), with one
//             accumulator per tile of 16 tokens; a lane fetches the hidden values of (block, token)
//             only when the token lists the block, which keeps the traffic from L2 at the size of the
//             supports instead of rows x all listed blocks.
// Hidden values travel as bf16 in [G][64][b] order; entries of tokens that do not list the block are
// neither written nor read.
#include "kernels.hpp"
#include "common.hpp"

namespace csk {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

constexpr int FW_MAXG = 1024;
constexpr int FW_ROWS = 64;                           // token rows of the hidden-value buffer per block
constexpr int GW_WAVES = 8, GW_THREADS = GW_WAVES * 64;
constexpr int GW_KC = GW_WAVES * 64;                  // columns of the token rows per staged chunk: 64 per wave
constexpr int GW_NT = 6;                              // tiles of 8 channels per pass of a workgroup
constexpr int GW_XROW = GW_KC + 8;                    // LDS row stride in elements: 16 bytes of padding
constexpr int DW_WAVES = 8;
constexpr int DW_UB = 3;                              // blocks in flight per wave

__device__ __forceinline__ bf16x8_t ldfrag(const uint16_t* p) { return *reinterpret_cast<const bf16x8_t*>(p); }
__device__ __forceinline__ bf16x8_t zfrag() {
    const uint4 z = make_uint4(0u, 0u, 0u, 0u);
    return *reinterpret_cast<const bf16x8_t*>(&z);
}

// Token masks per block (two words: bit t of word t / 32) and the ascending list of blocks used by at
// least one token.  Returns the number of listed blocks.
template <int NWAVES>
__device__ __forceinline__ int build_list64(const int32_t* __restrict__ support, int T, int k, int shared, int G,
                                            uint32_t* mlo, uint32_t* mhi, uint16_t* ulist, int* wcount) {
    constexpr int NTH = NWAVES * 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int g = tid; g < G; g += NTH) { mlo[g] = 0u; mhi[g] = 0u; }
    __syncthreads();
    const uint32_t all_lo = T >= 32 ? 0xFFFFFFFFu : ((1u << T) - 1u);
    const uint32_t all_hi = T >= 64 ? 0xFFFFFFFFu : (T > 32 ? ((1u << (T - 32)) - 1u) : 0u);
    const int total = shared ? k : T * k;
    for (int i = tid; i < total; i += NTH) {
        const int g = support[i];
        if (g >= 0 && g < G) {
            if (shared) { mlo[g] = all_lo; mhi[g] = all_hi; }
            else {
                const int t = i / k;
                if (t < 32) atomicOr(&mlo[g], 1u << t); else atomicOr(&mhi[g], 1u << (t - 32));
            }
        }
    }
    __syncthreads();
    int base = 0;
    for (int g0 = 0; g0 < G; g0 += NTH) {
        const int g = g0 + tid;
        const bool used = g < G && (mlo[g] | mhi[g]) != 0u;
        const unsigned long long bal = __ballot(used);
        if (lane == 0) wcount[wave] = __popcll(bal);
        __syncthreads();
        int off = base, tot = 0;
        for (int w = 0; w < NWAVES; ++w) { const int c = wcount[w]; if (w < wave) off += c; tot += c; }
        if (used) ulist[off + __popcll(bal & ((1ull << lane) - 1ull))] = (uint16_t)g;
        base += tot;
        __syncthreads();
    }
    return base;
}

template <int TT>
__global__ __launch_bounds__(GW_THREADS)
void ffn_gateup_wide(const uint16_t* __restrict__ Wg, const uint16_t* __restrict__ Wu, int d, int G, int b,
                     const uint16_t* __restrict__ x, int T, const int32_t* __restrict__ support, int k, int shared,
                     uint16_t* __restrict__ hbuf, uint32_t* __restrict__ list_out) {
    __shared__ uint32_t mlo[FW_MAXG], mhi[FW_MAXG];
    __shared__ uint16_t ulist[FW_MAXG];
    __shared__ int wcount[GW_WAVES];
    // token rows of one chunk, double buffered; the same memory holds the waves' partial tiles at the end of a pass
    __shared__ __attribute__((aligned(16))) uint16_t xs[2][TT * 16 * GW_XROW];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 15, kg = lane >> 4;

    // staging of the token rows: a chunk is TT*16 rows x GW_KC columns, in pieces of 16 bytes
    constexpr int PPR = GW_KC / 8;                                     // pieces per row
    constexpr int XP = (TT * 16 * PPR + GW_THREADS - 1) / GW_THREADS;  // pieces per thread
    uint4 xr[XP];
    auto x_fetch = [&](int chunk) {
#pragma unroll
        for (int p = 0; p < XP; ++p) {
            const int id = tid + p * GW_THREADS, row = id / PPR, piece = id % PPR;
            const bool ok = id < TT * 16 * PPR && row < T && chunk * GW_KC + piece * 8 < d;
            xr[p] = ok ? *reinterpret_cast<const uint4*>(x + (size_t)row * d + chunk * GW_KC + piece * 8) : make_uint4(0u, 0u, 0u, 0u);
        }
    };
    auto x_stash = [&](int buf) {
#pragma unroll
        for (int p = 0; p < XP; ++p) {
            const int id = tid + p * GW_THREADS, row = id / PPR, piece = id % PPR;
            if (id < TT * 16 * PPR) *reinterpret_cast<uint4*>(&xs[buf][row * GW_XROW + piece * 8]) = xr[p];
        }
    };
    x_fetch(0);                                       // in flight while the list is built

    const int nblocks = build_list64<GW_WAVES>(support, T, k, shared, G, mlo, mhi, ulist, wcount);
    // the down kernel takes the list and the masks from here: [0] count, [1 + i] block of slot i,
    // [1 + FW_MAXG + i] and [1 + 2 FW_MAXG + i] the two words of its token mask
    if (blockIdx.x == 0) {
        if (tid == 0) list_out[0] = (uint32_t)nblocks;
        for (int i = tid; i < nblocks; i += GW_THREADS) {
            const uint32_t g = ulist[i];
            list_out[1 + i] = g;
            list_out[1 + FW_MAXG + i] = mlo[g];
            list_out[1 + 2 * FW_MAXG + i] = mhi[g];
        }
    }
    // this workgroup's piece of the channel range, in passes of GW_NT tiles of 8 channels.  All waves work
    // on the same tiles and split the reduction index: within a chunk of GW_KC columns wave w takes
    // columns 64 w .. 64 w + 63, so that the workgroup as a whole reads 1 KB of consecutive addresses of
    // every weight row per chunk.
    const long F = (long)nblocks * b;
    const int f_lo = (int)((long)blockIdx.x * F / gridDim.x), f_hi = (int)((long)(blockIdx.x + 1) * F / gridDim.x);
    const int nchunks = (d + GW_KC - 1) / GW_KC;
    for (int f0 = f_lo; f0 < f_hi; f0 += GW_NT * 8) {
        // rows of this lane: tile nt, channel f0 + 8 nt + (ln & 7); lanes 0-7 of a 16-lane row take the
        // gate matrix, lanes 8-15 the up matrix
        const uint16_t* rp[GW_NT];
        bool row_ok[GW_NT];
#pragma unroll
        for (int nt = 0; nt < GW_NT; ++nt) {
            const int f = f0 + 8 * nt + (ln & 7);
            row_ok[nt] = f < f_hi;
            const int slot = row_ok[nt] ? f / b : 0;
            const int ch = row_ok[nt] ? f - slot * b : 0;
            rp[nt] = (ln < 8 ? Wg : Wu) + ((size_t)ulist[slot] * b + ch) * d + wave * 64 + kg * 8;
        }
        // the weights of the next chunk are requested into the registers of the current one as soon as
        // the matrix instructions have consumed them
        bf16x8_t wb[GW_NT][2];
        auto w_fetch = [&](int s, int chunk) {
            const int col = chunk * GW_KC + wave * 64 + s * 32;
#pragma unroll
            for (int nt = 0; nt < GW_NT; ++nt)
                wb[nt][s] = (row_ok[nt] && col < d) ? ldfrag(rp[nt] + chunk * GW_KC + s * 32) : zfrag();
        };
        w_fetch(0, 0);
        w_fetch(1, 0);
        if (f0 != f_lo) x_fetch(0);
        __syncthreads();                               // everybody is done with the staging buffers
        x_stash(0);
        __syncthreads();
        f32x4_t acc[GW_NT][TT];
#pragma unroll
        for (int nt = 0; nt < GW_NT; ++nt)
#pragma unroll
            for (int mt = 0; mt < TT; ++mt) acc[nt][mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        for (int c = 0; c < nchunks; ++c) {
            const int buf = c & 1;
            if (c + 1 < nchunks) x_fetch(c + 1);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                bf16x8_t a[TT];
#pragma unroll
                for (int mt = 0; mt < TT; ++mt)
                    a[mt] = *reinterpret_cast<const bf16x8_t*>(&xs[buf][(mt * 16 + ln) * GW_XROW + wave * 64 + s * 32 + kg * 8]);
#pragma unroll
                for (int nt = 0; nt < GW_NT; ++nt)
#pragma unroll
                    for (int mt = 0; mt < TT; ++mt)
                        acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mt], wb[nt][s], acc[nt][mt], 0, 0, 0);
                if (c + 1 < nchunks) w_fetch(s, c + 1);
            }
            if (c + 1 < nchunks) x_stash(buf ^ 1);
            __syncthreads();
        }
        // the waves' partial tiles are summed through LDS, one tile of 8 channels (x TT token tiles) at a time.
        // Element e = lane*4 + i of a 16 x 16 tile is (token 4*(lane/16)+i, column lane%16); columns 0-7 are
        // gate channels, 8-15 the matching up channels (32 elements further).
        float* red = reinterpret_cast<float*>(&xs[0][0]);              // [GW_WAVES][TT][256]
#pragma unroll
        for (int nt = 0; nt < GW_NT; ++nt) {
            if (f0 + 8 * nt < f_hi) {                                  // uniform over the workgroup
#pragma unroll
                for (int mt = 0; mt < TT; ++mt)
                    *reinterpret_cast<f32x4_t*>(&red[(wave * TT + mt) * 256 + lane * 4]) = acc[nt][mt];
                __syncthreads();
                for (int e = tid; e < TT * 256; e += GW_THREADS) {
                    const int mt = e >> 8, r = e & 255, col = (r >> 2) & 15;
                    const int f = f0 + 8 * nt + col;
                    if (col < 8 && f < f_hi) {
                        float sg = 0.f, su = 0.f;
#pragma unroll
                        for (int w = 0; w < GW_WAVES; ++w) { sg += red[(w * TT + mt) * 256 + r]; su += red[(w * TT + mt) * 256 + r + 32]; }
                        const int slot = f / b, ch = f - slot * b, g = ulist[slot];
                        const int tok = mt * 16 + 4 * (r >> 6) + (r & 3);
                        const bool uses = tok < 32 ? ((mlo[g] >> tok) & 1u) : ((mhi[g] >> (tok - 32)) & 1u);
                        if (tok < T && uses) hbuf[((size_t)g * FW_ROWS + tok) * b + ch] = f32_to_bf16(sg / (1.0f + __expf(-sg)) * su);
                    }
                }
                __syncthreads();
            }
        }
    }
}

template <int TT>
__global__ __launch_bounds__(DW_WAVES * 64)
void ffn_down_wide(const uint16_t* __restrict__ Wd, int d, int G, int b, const uint16_t* __restrict__ hbuf,
                   int T, const uint32_t* __restrict__ list_in, uint16_t* __restrict__ out) {
    __shared__ uint16_t ulist[FW_MAXG];
    __shared__ uint32_t ulo[FW_MAXG], uhi[FW_MAXG];
    __shared__ float red[DW_WAVES][TT * 256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < G; i += DW_WAVES * 64) {
        ulist[i] = (uint16_t)list_in[1 + i];
        ulo[i] = list_in[1 + FW_MAXG + i];
        uhi[i] = list_in[1 + 2 * FW_MAXG + i];
    }
    const int nblocks = min((int)list_in[0], G);
    const int ln = lane & 15, kg = lane >> 4;
    const int ksteps = b >> 5;
    const int ntiles = (d + 15) >> 4;
    __syncthreads();
    for (int tile = blockIdx.x; tile < ntiles; tile += (int)gridDim.x) {
        const int col0 = tile * 16;
        const bool row_ok = col0 + ln < d;
        f32x4_t acc[TT];
#pragma unroll
        for (int mt = 0; mt < TT; ++mt) acc[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        for (int u0 = wave; u0 < nblocks; u0 += DW_WAVES * DW_UB) {
            for (int ks = 0; ks < ksteps; ks += 2) {
                bf16x8_t wa[DW_UB][2], hb[DW_UB][TT][2];
#pragma unroll
                for (int q = 0; q < DW_UB; ++q) {
                    const int u = u0 + q * DW_WAVES;
                    const bool in_list = u < nblocks;
                    const int g = in_list ? ulist[u] : 0;
                    const uint32_t lo = in_list ? ulo[u] : 0u, hi = in_list ? uhi[u] : 0u;
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const bool ok = in_list && ks + e < ksteps;
                        const int ch = (ks + e) * 32 + kg * 8;
                        wa[q][e] = (ok && row_ok) ? ldfrag(Wd + ((size_t)g * d + col0 + ln) * b + ch) : zfrag();
#pragma unroll
                        for (int mt = 0; mt < TT; ++mt) {
                            const int tok = mt * 16 + ln;
                            const bool uses = mt < 2 ? ((lo >> (tok & 31)) & 1u) : ((hi >> (tok & 31)) & 1u);
                            hb[q][mt][e] = (ok && uses && tok < T) ? ldfrag(hbuf + ((size_t)g * FW_ROWS + tok) * b + ch) : zfrag();
                        }
                    }
                }
#pragma unroll
                for (int q = 0; q < DW_UB; ++q)
#pragma unroll
                    for (int e = 0; e < 2; ++e)
#pragma unroll
                        for (int mt = 0; mt < TT; ++mt)
                            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[q][e], hb[q][mt][e], acc[mt], 0, 0, 0);
            }
        }
#pragma unroll
        for (int mt = 0; mt < TT; ++mt) *reinterpret_cast<f32x4_t*>(&red[wave][mt * 256 + lane * 4]) = acc[mt];
        __syncthreads();
        // element e = lane*4 + i of tile mt is (output column 4*(lane/16)+i, token 16 mt + lane%16)
        for (int e = tid; e < TT * 256; e += DW_WAVES * 64) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < DW_WAVES; ++w) s += red[w][e];
            const int mt = e >> 8, r = e & 255;
            const int col = col0 + 4 * (r >> 6) + (r & 3), tok = mt * 16 + ((r >> 2) & 15);
            if (tok < T && col < d) out[(size_t)tok * d + col] = f32_to_bf16(s);
        }
        __syncthreads();                               // red[] is reused by the next tile
    }
}

bool ffn_wide_ok(const FfnArgs& a) {
    return a.dtype == 1 && !a.shared && a.T > 16 && a.T <= FW_ROWS && a.G <= FW_MAXG && (a.d % 32) == 0 &&
           (a.b % 32) == 0;
}

size_t ffn_wide_scratch_bytes(const FfnArgs& a) {
    return (size_t)a.G * FW_ROWS * a.b * sizeof(uint16_t) + (3 * FW_MAXG + 4) * sizeof(uint32_t);
}

hipError_t launch_ffn_wide(const FfnArgs& a, hipStream_t s) {
    uint16_t* hbuf = reinterpret_cast<uint16_t*>(a.scratch);
    uint32_t* list = reinterpret_cast<uint32_t*>(hbuf + (size_t)a.G * FW_ROWS * a.b);
    const int union_max = a.T * a.k < a.G ? a.T * a.k : a.G;
    long grid = (long)union_max * a.b / 8;             // at least one tile of 8 channels per workgroup
    if (grid > 256) grid = 256;
    if (grid < 1) grid = 1;
    int dgrid = (a.d + 15) / 16;
    if (dgrid > 256) dgrid = 256;
    const int tt = (a.T + 15) / 16;
#define CS_WIDE(TTV) do { \
        hipLaunchKernelGGL((ffn_gateup_wide<TTV>), dim3((unsigned)grid), dim3(GW_THREADS), 0, s, (const uint16_t*)a.Wg, \
                           (const uint16_t*)a.Wu, a.d, a.G, a.b, (const uint16_t*)a.x, a.T, a.support, a.k, a.shared, hbuf, list); \
        hipLaunchKernelGGL((ffn_down_wide<TTV>), dim3(dgrid), dim3(DW_WAVES * 64), 0, s, (const uint16_t*)a.Wd, a.d, a.G, \
                           a.b, hbuf, a.T, list, (uint16_t*)a.out); } while (0)
    if (tt <= 2) CS_WIDE(2); else if (tt == 3) CS_WIDE(3); else CS_WIDE(4);
#undef CS_WIDE
    return hipGetLastError();
}

}  // namespace csk
