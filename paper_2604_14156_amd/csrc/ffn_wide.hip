// Block-sparse gated feed-forward layer for token-adaptive batches of 17 to 64 rows (paper Sec. 5: every
// token has its own support; Sec. 7: the units are blocks of contiguous channels), bf16.
//
// Like the path for up to 16 rows, the layer is bound by the memory system: every block listed by at
// least one token has to be read once, and 64 rows per weight byte are far from filling the matrix cores.
// What changes against the 16-row kernels is where the token rows live.  Sixteen rows fit into the
// registers of the waves that split the reduction index; sixty-four do not (they would take the whole
// register file of a compute unit).  So here
//   gate/up : the channels of all listed blocks form one range cut into gridDim.x equal pieces, so every
//             workgroup streams the same number of bytes, and a workgroup's piece is cut once more
//             among its waves, in whole tiles.  A wave owns a tile of 8 channels (8 gate rows + 8 up rows) over the
//             whole reduction index: its accumulators (one per tile of 16 tokens) are final, nothing
//             is summed across waves.  Weights go global -> registers -> matrix core; the registers
//             of a k-step are refilled with the next chunk's weights right after use, so every load
//             has a chunk's time to arrive.  The token rows are staged chunk by chunk (512 columns)
//             through LDS, double buffered and shared by the waves, and come from L2 (every
//             workgroup reads the same rows).  The first chunk of weights is requested before the
//             supports have arrived when their union can be guessed.
//   down    : as for 16 rows (a workgroup owns 16 output columns, waves split the blocks), with one
//             accumulator per tile of 16 tokens; a lane fetches the hidden values of (block, token)
//             only when the token lists the block, which keeps the traffic from L2 at the size of the
//             supports instead of rows x all listed blocks.
// Hidden values travel as bf16 in [G][64][b] order; entries of tokens that do not list the block are
// neither written nor read.
#include "kernels.hpp"
#include "common.hpp"
#include <type_traits>

namespace csk {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

constexpr int FW_MAXG = 1024;
constexpr int FW_ROWS = 64;                           // token rows of the hidden-value buffer per block
constexpr int GW_WAVES = 8, GW_THREADS = GW_WAVES * 64;
constexpr int GW_KC = 512;                            // columns of the token rows per staged chunk
// LDS serves a 16-byte read per lane sixteen lanes at a time, and the sixteen are lanes 0-7 with 24-31, 8-15 with
// 16-23 (likewise in the upper half of the wave); they must fall into sixteen different 16-byte columns of the
// 256-byte bank row or the read takes twice as long (measured).  For fragment reads (lane = row % 16 + 16 * piece)
// that means: a row stride of 32 bytes modulo 256 where rows may be padded, and for the unpadded 128-byte rows of
// the turning tiles the piece index XORed with (row & 6).
constexpr int GW_XROW = GW_KC + 16;                   // LDS row stride in elements: 32 bytes of padding
constexpr int GW_TROW = 64;                           // row stride of a wave's turning tile in elements (one line, pieces swizzled)
constexpr int DW_WAVES = 16;
constexpr int DW_UB = 1;                              // blocks in flight per wave (16 x 1 beats 8 x 3 by 2 us at 32 rows, equal at 64)

__device__ __forceinline__ bf16x8_t ldfrag(const uint16_t* p) { return *reinterpret_cast<const bf16x8_t*>(p); }
__device__ __forceinline__ bf16x8_t ldfrag_once(const uint16_t* p) {       // read once, whole lines per load
    return __builtin_nontemporal_load(reinterpret_cast<const bf16x8_t*>(p));
}
// Lanes of one wave hand data to each other through LDS without a workgroup barrier.  The hardware runs a
// wave's LDS operations in program order; the compiler, which otherwise may treat what a thread has not
// written itself as unchanged, is told by this fence that the other lanes' stores are to be seen.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__device__ __forceinline__ bf16x8_t zfrag() {
    const uint4 z = make_uint4(0u, 0u, 0u, 0u);
    return *reinterpret_cast<const bf16x8_t*>(&z);
}

// Token masks per block (two words: bit t of word t / 32) and the ascending list of blocks used by at
// least one token.  Returns the number of listed blocks.  `pre` holds support[tid + q * NTH] (or -1 past
// the end) for q < NPRE, fetched by the caller ahead of its other loads: loads return in order, so an
// entry requested after the first weights would arrive behind them.
template <int NWAVES, int NPRE>
__device__ __forceinline__ int build_list64(const int32_t* __restrict__ support, const int (&pre)[NPRE], int T, int k,
                                            int shared, int G, uint32_t* mlo, uint32_t* mhi, uint16_t* ulist, int* wcount) {
    constexpr int NTH = NWAVES * 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int g = tid; g < G; g += NTH) { mlo[g] = 0u; mhi[g] = 0u; }
    __syncthreads();
    const uint32_t all_lo = T >= 32 ? 0xFFFFFFFFu : ((1u << T) - 1u);
    const uint32_t all_hi = T >= 64 ? 0xFFFFFFFFu : (T > 32 ? ((1u << (T - 32)) - 1u) : 0u);
    const int total = shared ? k : T * k;
    auto mark = [&](int i, int g) {
        if (g >= 0 && g < G) {
            if (shared) { mlo[g] = all_lo; mhi[g] = all_hi; }
            else {
                // i / k without the integer division: exact, since the token index stays below 64 and k
                // below 2^10, so (i + 0.5) / k keeps 2^-11 away from the next integer
                const int t = (int)__fdividef((float)i + 0.5f, (float)k);
                if (t < 32) atomicOr(&mlo[g], 1u << t); else atomicOr(&mhi[g], 1u << (t - 32));
            }
        }
    };
#pragma unroll
    for (int q = 0; q < NPRE; ++q) { const int i = tid + q * NTH; if (i < total) mark(i, pre[q]); }
    for (int i = tid + NPRE * NTH; i < total; i += NTH) mark(i, support[i]);
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

// `dense` is the host's guess that the union of the supports is all G blocks (many rows, each listing a
// good share of the blocks).  The weights of the first chunk are then requested at kernel entry for the
// channel range that guess implies, a full memory round trip before the supports have come in and the
// list is known; if the list turns out shorter, the range is recomputed and the loads are issued again
// (the dropped ones were in bounds whatever the supports say).
template <int TT>
__global__ __launch_bounds__(GW_THREADS)
void ffn_gateup_wide(const uint16_t* __restrict__ Wg, const uint16_t* __restrict__ Wu, int d, int G, int b,
                     const uint16_t* __restrict__ x, int T, const int32_t* __restrict__ support, int k, int shared,
                     int dense, uint16_t* __restrict__ hbuf, uint32_t* __restrict__ list_out) {
    __shared__ uint32_t mlo[FW_MAXG], mhi[FW_MAXG];
    __shared__ uint16_t ulist[FW_MAXG];
    __shared__ int wcount[GW_WAVES];
    __shared__ __attribute__((aligned(16))) uint16_t xs[2][TT * 16 * GW_XROW];   // token rows of one chunk, double buffered
    __shared__ __attribute__((aligned(16))) uint16_t turns[GW_WAVES][16 * GW_TROW];   // per wave: 16 weight rows x 128 bytes, pieces swizzled
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 15, kg = lane >> 4;

    // staging of the token rows: a chunk is TT*16 rows x GW_KC columns, in pieces of 16 bytes
    constexpr int PPR = GW_KC / 8;                                     // pieces per row
    constexpr int XP = (TT * 16 * PPR + GW_THREADS - 1) / GW_THREADS;  // pieces per thread
    static_assert((TT * 16 * PPR) % GW_THREADS == 0, "every thread stages the same number of pieces");
    uint4 xr[XP];
    // rows past the last token repeat it: their products land in accumulator rows that are never stored
    uint32_t xoff[XP];
#pragma unroll
    for (int p = 0; p < XP; ++p) {
        const int id = tid + p * GW_THREADS, row = id / PPR, piece = id % PPR;
        xoff[p] = (uint32_t)min(row, T - 1) * (uint32_t)d + (uint32_t)piece * 8u;
    }
    auto x_fetch = [&](int chunk) {
        if ((chunk + 1) * GW_KC <= d) {                // uniform: a whole chunk
#pragma unroll
            for (int p = 0; p < XP; ++p) xr[p] = *reinterpret_cast<const uint4*>(x + xoff[p] + (uint32_t)(chunk * GW_KC));
        } else {
#pragma unroll
            for (int p = 0; p < XP; ++p) {
                const int piece = (tid + p * GW_THREADS) % PPR;
                xr[p] = chunk * GW_KC + piece * 8 < d ? *reinterpret_cast<const uint4*>(x + xoff[p] + (uint32_t)(chunk * GW_KC))
                                                      : make_uint4(0u, 0u, 0u, 0u);
            }
        }
    };
    auto x_stash = [&](int buf) {
#pragma unroll
        for (int p = 0; p < XP; ++p) {
            const int id = tid + p * GW_THREADS, row = id / PPR, piece = id % PPR;
            *reinterpret_cast<uint4*>(&xs[buf][row * GW_XROW + piece * 8]) = xr[p];
        }
    };
    constexpr int NPRE = 8;
    int pre[NPRE];
    {
        const int total = shared ? k : T * k;
#pragma unroll
        for (int q = 0; q < NPRE; ++q) { const int i = tid + q * GW_THREADS; pre[q] = i < total ? support[i] : -1; }
    }

    // The channels of the listed blocks form one range cut into gridDim.x equal pieces, and a workgroup's
    // piece into GW_WAVES equal pieces: wave w owns channels [w_lo, w_hi) and works through them in tiles
    // of 8 (8 gate rows + 8 up rows = the 16 columns of a matrix-core tile), all of the reduction index
    // per tile.  Weights are loaded as whole 128-byte lines with the non-temporal hint (eight lanes per row:
    // lane (lr, lc) takes piece lc of gate row c0 + lr and of up row c0 + lr for each pair of k-steps) and
    // turned into the two fragments of the pair through a per-wave LDS tile, as in the 16-row kernels:
    // fragment-order loads (16 rows x 64 bytes per instruction) fetch every line twice and lose 13 % of the
    // streaming rate.
    constexpr int KS = GW_KC / 32;                     // k-steps per chunk
    int w_lo = 0, w_hi = 0, npass = 0;
    auto set_range = [&](int nb) {
        const long F = (long)nb * b;
        const int f_lo = (int)((long)blockIdx.x * F / gridDim.x), f_hi = (int)((long)(blockIdx.x + 1) * F / gridDim.x);
        // whole tiles of 8 channels per wave: a wave with 6 of its 8 rows in use issues the same loads and
        // multiplies as a full one (43 channels per workgroup: five full waves and one with three rows
        // instead of seven waves with six rows; the waves left without rows still stage the token rows)
        const int cpw = ((f_hi - f_lo + GW_WAVES - 1) / GW_WAVES + 7) & ~7;
        w_lo = min(f_hi, f_lo + wave * cpw);
        w_hi = min(f_hi, w_lo + cpw);
        npass = (cpw + 7) >> 3;                        // the same for every wave of the workgroup
    };
    const int lr = lane >> 3, lc = lane & 7;           // as a loader: row of the half tile, 16-byte piece of the line
    // the loader's weight row of the current tile (same offset in Wg and Wu), at piece lc; a 32-bit element
    // offset from the uniform bases (the host sends larger weight arrays down another path), which is what
    // lets the instance with four token tiles keep everything in registers
    uint32_t wrow = 0;
    int my_g = 0, my_ch = 0;                           // the block and channel whose hidden values this lane stores
    bool my_ok = false;
    auto set_tile = [&](int c0, bool identity) {
        const int f = c0 + (ln & 7);
        my_ok = f < w_hi;
        const int fc = my_ok ? f : c0;                 // rows past the end repeat the first one; they are not stored
        const int slot = fc / b;
        my_ch = fc - slot * b;
        my_g = identity ? slot : (int)ulist[slot];
        const int fl = c0 + lr < w_hi ? c0 + lr : c0;
        const int lslot = fl / b;
        const int lg = identity ? lslot : (int)ulist[lslot];
        wrow = (uint32_t)((lg * b + (fl - lslot * b)) * d + lc * 8);
    };
    // The weights of a chunk as loaded: wb[2 p] the gate lines, wb[2 p + 1] the up lines of the pair of k-steps p.
    // In a chunk that runs past the last column the pieces beyond it are read at column 0 instead (in bounds)
    // and meet the zeros staged for the token rows.
    bf16x8_t wb[KS];
    auto w_fetch_all = [&](int chunk) {
#pragma unroll
        for (int pr = 0; pr < KS / 2; ++pr) {
            const int col = chunk * GW_KC + pr * 64;
            const uint32_t off = wrow + (uint32_t)(col + lc * 8 < d ? col : -lc * 8);
            wb[2 * pr] = ldfrag_once(Wg + off);
            wb[2 * pr + 1] = ldfrag_once(Wu + off);
        }
    };
    // lines -> fragments: lane (ln, kg) reads row ln (gate rows 0-7, up rows 8-15), piece 4 e + kg for k-step 2 p + e
    uint16_t* turn = turns[wave];
    uint16_t* turn_w = turn + lr * GW_TROW + ((lc ^ (lr & 6)) * 8);            // rows lr and 8 + lr share the swizzle
    const uint16_t* turn_r0 = turn + ln * GW_TROW + ((kg ^ (ln & 6)) * 8);
    const uint16_t* turn_r1 = turn + ln * GW_TROW + ((kg ^ (ln & 6) ^ 4) * 8);
    auto to_frags = [&](const bf16x8_t& gate_lines, const bf16x8_t& up_lines, bf16x8_t& f0, bf16x8_t& f1) {
        *reinterpret_cast<bf16x8_t*>(turn_w) = gate_lines;
        *reinterpret_cast<bf16x8_t*>(turn_w + 8 * GW_TROW) = up_lines;
        wave_lds_fence();
        f0 = *reinterpret_cast<const bf16x8_t*>(turn_r0);
        f1 = *reinterpret_cast<const bf16x8_t*>(turn_r1);
        wave_lds_fence();
    };
    // Chunks are taken in an order rotated by the workgroup's index (when all chunks are whole), so that the
    // workgroups do not all ask L2 for the same token rows at the same moment.
    const int nchunks = (d + GW_KC - 1) / GW_KC;
    const int nwhole = d / GW_KC;                      // chunks 0 .. nwhole - 1 are whole, one ragged chunk may follow
    const int rot = nwhole == nchunks ? (int)(blockIdx.x % (unsigned)nchunks) : 0;
    auto chunk_of = [&](int i) { const int c = i + rot; return c >= nchunks ? c - nchunks : c; };

    // issued by every lane whatever `dense` says (a wave without a share, or a call whose union is not
    // guessed, reads rows it will drop): the number of loads in flight is then known at compile time, and
    // the wait for the support entries does not have to cover the weights as well
    x_fetch(chunk_of(0));
    set_range(G);
    set_tile(min(w_lo, G * b - 1), true);
    w_fetch_all(chunk_of(0));
    const int nblocks = build_list64<GW_WAVES, NPRE>(support, pre, T, k, shared, G, mlo, mhi, ulist, wcount);
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
    const bool guessed = dense && nblocks == G;        // an ascending list of all G blocks is the identity
    if (!guessed) set_range(nblocks);
    for (int pass = 0; pass < npass; ++pass) {
        const int c0 = w_lo + 8 * pass;
        const bool busy = c0 < w_hi;                   // uniform over the wave
        if (busy && !(pass == 0 && guessed)) { set_tile(c0, false); w_fetch_all(chunk_of(0)); }
        if (pass != 0) x_fetch(chunk_of(0));
        __syncthreads();                               // everybody is done with the staging buffers
        x_stash(0);
        __syncthreads();
        f32x4_t acc[TT];
#pragma unroll
        for (int mt = 0; mt < TT; ++mt) acc[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        // One chunk (the i-th in this workgroup's order): the token rows of the next chunk are requested
        // first, then the k-steps run: the token fragments of k-step s + 1 are read from LDS before the
        // matrix instructions of k-step s are issued (the scheduling fences keep that order, so no matrix
        // instruction waits for a read issued just before it), and the registers of a k-step take the
        // next chunk's weights as soon as they are free, so every fragment has a chunk's time to arrive.
        // NEXT says what follows the chunk (0 nothing, 1 a whole chunk, 2 a ragged one) at compile time:
        // the loop over the whole chunks is free of branches, and the other two cases stand after it.
        auto chunk_step = [&](int i, auto next) {
            constexpr int NEXT = decltype(next)::value;
            const int buf = i & 1;
            const int cn = chunk_of(i + 1);
            if (NEXT != 0) x_fetch(cn);
            if (busy) {
                const uint32_t wnext = wrow + (uint32_t)(cn * GW_KC);
                const uint16_t* xb = &xs[buf][ln * GW_XROW + kg * 8];
                bf16x8_t a[2][TT];
#pragma unroll
                for (int mt = 0; mt < TT; ++mt) a[0][mt] = *reinterpret_cast<const bf16x8_t*>(xb + mt * 16 * GW_XROW);
#pragma unroll
                for (int pr = 0; pr < KS / 2; ++pr) {
                    bf16x8_t f[2];
                    to_frags(wb[2 * pr], wb[2 * pr + 1], f[0], f[1]);
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const int s = 2 * pr + e;
                        if (s + 1 < KS) {
#pragma unroll
                            for (int mt = 0; mt < TT; ++mt)
                                a[(s + 1) & 1][mt] = *reinterpret_cast<const bf16x8_t*>(xb + mt * 16 * GW_XROW + (s + 1) * 32);
                        }
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int mt = 0; mt < TT; ++mt)
                            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[s & 1][mt], f[e], acc[mt], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (NEXT == 1) {
                        wb[2 * pr] = ldfrag_once(Wg + wnext + pr * 64);
                        wb[2 * pr + 1] = ldfrag_once(Wu + wnext + pr * 64);
                    }
                    if (NEXT == 2) {
                        const int col = cn * GW_KC + pr * 64;
                        const uint32_t off = wrow + (uint32_t)(col + lc * 8 < d ? col : -lc * 8);
                        wb[2 * pr] = ldfrag_once(Wg + off);
                        wb[2 * pr + 1] = ldfrag_once(Wu + off);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (NEXT != 0) x_stash(buf ^ 1);
            __syncthreads();
        };
        int i = 0;
        for (; i + 1 < nwhole; ++i) chunk_step(i, std::integral_constant<int, 1>{});
        if (nwhole < nchunks) {
            if (nwhole > 0) { chunk_step(i, std::integral_constant<int, 2>{}); ++i; }
            chunk_step(i, std::integral_constant<int, 0>{});
        } else {
            chunk_step(i, std::integral_constant<int, 0>{});
        }
        // Element i of a lane's accumulator is (token 16 mt + 4 (lane / 16) + i, column lane % 16); columns 0-7
        // are the gate channels, 8-15 the matching up channels, eight lanes further.
        if (busy) {
            const uint32_t lo = mlo[my_g], hi = mhi[my_g];
#pragma unroll
            for (int mt = 0; mt < TT; ++mt) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float mine = acc[mt][e];
                    const float other = __shfl_xor(mine, 8);
                    const int tok = mt * 16 + 4 * kg + e;
                    const bool uses = mt < 2 ? ((lo >> (tok & 31)) & 1u) : ((hi >> (tok & 31)) & 1u);
                    if (ln < 8 && my_ok && tok < T && uses)
                        hbuf[((size_t)my_g * FW_ROWS + tok) * b + my_ch] = f32_to_bf16(mine / (1.0f + __expf(-mine)) * other);
                }
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
    __shared__ __attribute__((aligned(16))) uint16_t turns[DW_WAVES][16 * GW_TROW];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint16_t* turn = turns[wave];
    const int lr = lane >> 3, lc = lane & 7;           // as a loader: row of the half tile, 16-byte piece of the line
    for (int i = tid; i < G; i += DW_WAVES * 64) {
        ulist[i] = (uint16_t)list_in[1 + i];
        ulo[i] = list_in[1 + FW_MAXG + i];
        uhi[i] = list_in[1 + 2 * FW_MAXG + i];
    }
    const int nblocks = min((int)list_in[0], G);
    const int ln = lane & 15, kg = lane >> 4;
    uint16_t* turn_w = turn + lr * GW_TROW + ((lc ^ (lr & 6)) * 8);
    const uint16_t* turn_r0 = turn + ln * GW_TROW + ((kg ^ (ln & 6)) * 8);
    const uint16_t* turn_r1 = turn + ln * GW_TROW + ((kg ^ (ln & 6) ^ 4) * 8);
    const int ksteps = b >> 5;
    const int ntiles = (d + 15) >> 4;
    __syncthreads();
    for (int tile = blockIdx.x; tile < ntiles; tile += (int)gridDim.x) {
        const int col0 = tile * 16;
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
                        // Weights come as whole lines, read once: load e is 64 channels of output rows 8 e .. 8 e + 7.
                        const int wrow = col0 + 8 * e + lr, wch = ks * 32 + lc * 8;
                        wa[q][e] = (in_list && wch < b && wrow < d) ? ldfrag_once(Wd + ((size_t)g * d + wrow) * b + wch) : zfrag();
#pragma unroll
                        for (int mt = 0; mt < TT; ++mt) {
                            const int tok = mt * 16 + ln;
                            const bool uses = mt < 2 ? ((lo >> (tok & 31)) & 1u) : ((hi >> (tok & 31)) & 1u);
                            hb[q][mt][e] = (ok && uses && tok < T) ? ldfrag(hbuf + ((size_t)g * FW_ROWS + tok) * b + ch) : zfrag();
                        }
                    }
                }
#pragma unroll
                for (int q = 0; q < DW_UB; ++q) {
                    // The wave's tile turns the two line loads into the fragments of the two k-steps.
                    bf16x8_t f[2];
                    *reinterpret_cast<bf16x8_t*>(turn_w) = wa[q][0];
                    *reinterpret_cast<bf16x8_t*>(turn_w + 8 * GW_TROW) = wa[q][1];
                    wave_lds_fence();
                    f[0] = *reinterpret_cast<const bf16x8_t*>(turn_r0);
                    f[1] = *reinterpret_cast<const bf16x8_t*>(turn_r1);
                    wave_lds_fence();
#pragma unroll
                    for (int e = 0; e < 2; ++e)
#pragma unroll
                        for (int mt = 0; mt < TT; ++mt)
                            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[e], hb[q][mt][e], acc[mt], 0, 0, 0);
                }
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
           (a.b % 32) == 0 && (long long)a.G * a.b * a.d < (1LL << 31);   // 32-bit element offsets in the gate/up kernel
}

size_t ffn_wide_scratch_bytes(const FfnArgs& a) {
    return (size_t)a.G * FW_ROWS * a.b * sizeof(uint16_t) + (3 * FW_MAXG + 4) * sizeof(uint32_t);
}

hipError_t launch_ffn_wide(const FfnArgs& a, hipStream_t s) {
    uint16_t* hbuf = reinterpret_cast<uint16_t*>(a.scratch);
    uint32_t* list = reinterpret_cast<uint32_t*>(hbuf + (size_t)a.G * FW_ROWS * a.b);
    const int union_max = a.T * a.k < a.G ? a.T * a.k : a.G;
    long grid = (long)union_max * a.b / 8;             // at least one tile of 8 channels per workgroup
    // every block is then listed by some row, almost surely (or the caller has said so, or the opposite)
    const int dense = a.union_hint == 1 || (a.union_hint == 0 && (long)a.T * a.k >= 4L * a.G);
    if (grid > 256) grid = 256;
    if (grid < 1) grid = 1;
    int dgrid = (a.d + 15) / 16;
    if (dgrid > 256) dgrid = 256;
    const int tt = (a.T + 15) / 16;
#define CS_WIDE(TTV) do { \
        hipLaunchKernelGGL((ffn_gateup_wide<TTV>), dim3((unsigned)grid), dim3(GW_THREADS), 0, s, (const uint16_t*)a.Wg, \
                           (const uint16_t*)a.Wu, a.d, a.G, a.b, (const uint16_t*)a.x, a.T, a.support, a.k, a.shared, dense, hbuf, list); \
        hipLaunchKernelGGL((ffn_down_wide<TTV>), dim3(dgrid), dim3(DW_WAVES * 64), 0, s, (const uint16_t*)a.Wd, a.d, a.G, \
                           a.b, hbuf, a.T, list, (uint16_t*)a.out); } while (0)
    if (tt <= 2) CS_WIDE(2); else if (tt == 3) CS_WIDE(3); else CS_WIDE(4);
#undef CS_WIDE
    return hipGetLastError();
}

}  // namespace csk
