// Block-sparse gated feed-forward layer restricted to a recovered support
// (masked execution of paper Sec. 3 with the block structure of Sec. 7):
//   out[t] = sum_{g in S_t} Wd_g ( silu(Wg_g x_t) * (Wu_g x_t) ).
// Only the weight blocks named by the support are read.
#include "kernels.hpp"
#include "common.hpp"

namespace csk {

// ---------------------------------------------------------------------------
// Generic path (any element type, any T, shared or per-token supports).
// Phase 1: one workgroup per (token, support slot); a wavefront owns a channel and
//          reduces its two dot products over the 64 lanes.
// Phase 2: one thread per output column; the token's k*b hidden values sit in LDS.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256)
void ffn_hidden_generic(const T* __restrict__ Wg, const T* __restrict__ Wu, int d, int G, int b,
                        const T* __restrict__ x, const int32_t* __restrict__ support, int k, int shared,
                        float* __restrict__ hid) {
    const int j = blockIdx.x, t = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = support[shared ? j : t * k + j];
    float* h = hid + ((size_t)t * k + j) * b;
    if (g < 0 || g >= G) {
        for (int c = threadIdx.x; c < b; c += 256) h[c] = 0.f;
        return;
    }
    const T* xr = x + (size_t)t * d;
    for (int c = wave; c < b; c += 4) {
        const T* wg = Wg + ((size_t)g * b + c) * d;
        const T* wu = Wu + ((size_t)g * b + c) * d;
        float sg = 0.f, su = 0.f;
        for (int e = lane * 8; e < d; e += 512) {
            float xv[8], a[8], u[8];
            load8(xr + e, xv); load8(wg + e, a); load8(wu + e, u);
#pragma unroll
            for (int i = 0; i < 8; ++i) { sg += a[i] * xv[i]; su += u[i] * xv[i]; }
        }
        sg = wave_sum(sg); su = wave_sum(su);
        if (lane == 0) h[c] = sg / (1.0f + expf(-sg)) * su;
    }
}

template <typename T>
__global__ __launch_bounds__(256)
void ffn_down_generic(const T* __restrict__ Wd, int d, int G, int b,
                      const int32_t* __restrict__ support, int k, int shared,
                      const float* __restrict__ hid, T* __restrict__ out) {
    extern __shared__ float hs[];                  // [k][b]
    const int t = blockIdx.y;
    const int col = blockIdx.x * 256 + threadIdx.x;
    const float* h = hid + (size_t)t * k * b;
    for (int i = threadIdx.x; i < k * b; i += 256) hs[i] = h[i];
    __syncthreads();
    if (col >= d) return;
    float acc = 0.f;
    for (int j = 0; j < k; ++j) {
        const int g = support[shared ? j : t * k + j];
        if (g < 0 || g >= G) continue;
        const T* w = Wd + ((size_t)g * d + col) * b;
        for (int c = 0; c < b; c += 8) {
            float wv[8];
            load8(w + c, wv);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc += wv[i] * hs[j * b + c + i];
        }
    }
    store1(out + (size_t)t * d + col, acc);
}

template <typename T>
static hipError_t run_generic(const FfnArgs& a, hipStream_t s) {
    float* hid = reinterpret_cast<float*>(a.scratch);
    hipLaunchKernelGGL((ffn_hidden_generic<T>), dim3(a.k, a.T), dim3(256), 0, s,
                       (const T*)a.Wg, (const T*)a.Wu, a.d, a.G, a.b, (const T*)a.x, a.support, a.k, a.shared, hid);
    const size_t hs_bytes = (size_t)a.k * a.b * sizeof(float);
    if (hs_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(ffn_down_generic<T>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)hs_bytes);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((ffn_down_generic<T>), dim3((a.d + 255) / 256, a.T), dim3(256), hs_bytes, s,
                       (const T*)a.Wd, a.d, a.G, a.b, a.support, a.k, a.shared, hid, (T*)a.out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Decode path, bf16, up to 16 tokens per launch (token-adaptive supports, Sec. 5).
//
// The layer is bandwidth bound: every active weight block must be read once, and
// the arithmetic per byte is tiny.  The matrix cores are used only because they
// consume a 16-byte weight fragment per lane without any unpacking, which keeps
// the vector ALUs out of the way of the loads; the 16-token operand is padded with
// zero rows.
//
// gate/up kernel: a workgroup of 16 waves walks over (active block, 8-channel
//   chunk) items.  Wave w owns the input columns of k-steps w, w+16, ... (32
//   columns each) and keeps that slice of all 16 token rows in registers for the
//   whole kernel; per item it streams the matching slice of 8 gate rows and 8 up
//   rows (one 16x16 tile), and the 16 partial tiles are summed through LDS.
//   The loads of the next item are issued before the current tile is reduced.
//   A load instruction covers whole 128-byte lines (8 rows x 128 bytes: eight lanes
//   per row) and carries the non-temporal hint; a matrix-core fragment wants 16
//   rows x 64 bytes per instruction, so the wave turns two loads (8 gate rows, 8 up
//   rows) into the two fragments of a pair of k-steps through a small LDS tile of
//   its own.  Loading in fragment order instead costs 13 % of the streaming rate
//   (each line fetched by two instructions; measured on a read-only copy of the
//   access pattern: 32.8 against 28.5 us for the 178 MB of a call).
// down kernel: a workgroup owns 16 output columns; its waves split the active
//   blocks, each multiplying the block's [16 x b] slice of Wd (one contiguous
//   run of 16 rows) with the block's hidden values, then the waves are summed.
// Hidden values travel between the two kernels as bf16 in [G][16][b] order,
// already masked by "token t uses block g".
// ---------------------------------------------------------------------------
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

constexpr int FD_WAVES = 16;
constexpr int FD_THREADS = FD_WAVES * 64;
constexpr int FD_MAXG = 1024;
// Turning tiles: 16 rows of one 128-byte line.  LDS serves a 16-byte read per lane sixteen lanes at a time (lanes
// 0-7 with 24-31, 8-15 with 16-23, likewise in the upper half of the wave), and the sixteen must fall into
// different 16-byte columns of the 256-byte bank row or the read takes 1.6 times as long (measured).  A fragment
// read has lane = row + 16 * piece, so the rows are left unpadded and piece p of row r sits at p ^ (r & 6).
constexpr int FD_TROW = 64;                           // row stride of a wave's turning tile in elements
__device__ __forceinline__ int turn_at(int row, int piece) { return row * FD_TROW + ((piece ^ (row & 6)) << 3); }

__device__ __forceinline__ bf16x8_t load_frag(const uint16_t* p) {
    return *reinterpret_cast<const bf16x8_t*>(p);
}
// (Not read with the non-temporal hint, although every weight is read once: a fragment load takes 64 of a
// line's 128 bytes and the neighbouring k-step's load the rest; with the hint the two no longer share the
// fetch of the line, and both kernels get slower: 38.3 -> 40.9 us and 19.8 -> 21.8 us at 16 rows.)
// Weights are read once per call, whole lines per load: the non-temporal hint keeps them from displacing
// anything on their way (a plain streaming read gains a tenth with it on this device).
__device__ __forceinline__ bf16x8_t load_frag_once(const uint16_t* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const bf16x8_t*>(p));
}
// Lanes of one wave hand data to each other through LDS without a workgroup barrier.  The hardware runs a
// wave's LDS operations in program order; the compiler, which otherwise may treat what a thread has not
// written itself as unchanged, is told by this fence that the other lanes' stores are to be seen.
__device__ __forceinline__ void wave_fence_lds() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__device__ __forceinline__ bf16x8_t zero_frag() {
    const uint4 z = make_uint4(0u, 0u, 0u, 0u);
    return *reinterpret_cast<const bf16x8_t*>(&z);
}

// Token masks per block and the compacted list of blocks used by at least one token.
// mask[g] bit t = token t lists block g.  Returns the number of listed blocks.
// `pre` is support[threadIdx.x] (or -1 past the end), fetched by the caller ahead of its other loads:
// loads return in order, so a support entry requested after them would wait for all of them.
template <int NWAVES>
__device__ __forceinline__ int build_block_list(const int32_t* __restrict__ support, int pre, int T, int k, int shared, int G,
                                                uint32_t* mask, uint16_t* ulist, int* wcount) {
    constexpr int NTH = NWAVES * 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (shared || T == 1) {
        // one support for everything: the list is the support itself (entries are distinct by
        // contract; out-of-range entries are dropped), every row uses every listed block
        const uint32_t allbits = T >= 32 ? 0xFFFFFFFFu : ((1u << T) - 1u);
        int base = 0;
        for (int i0 = 0; i0 < k; i0 += NTH) {
            const int i = i0 + tid;
            const int g = i < k ? (i0 == 0 ? pre : support[i]) : -1;
            const bool used = g >= 0 && g < G;
            const unsigned long long bal = __ballot(used);
            if (lane == 0) wcount[wave] = __popcll(bal);
            __syncthreads();
            int off = base, tot = 0;
            for (int w = 0; w < NWAVES; ++w) { const int c = wcount[w]; if (w < wave) off += c; tot += c; }
            if (used) { ulist[off + __popcll(bal & ((1ull << lane) - 1ull))] = (uint16_t)g; mask[g] = allbits; }
            base += tot;
            __syncthreads();
        }
        return base;
    }
    for (int g = tid; g < G; g += NTH) mask[g] = 0u;
    __syncthreads();
    const int total = shared ? k : T * k;
    const uint32_t allbits = T >= 32 ? 0xFFFFFFFFu : ((1u << T) - 1u);
    for (int i = tid; i < total; i += NTH) {
        const int g = i == tid ? pre : support[i];
        if (g >= 0 && g < G) atomicOr(&mask[g], shared ? allbits : (1u << (i / k)));
    }
    __syncthreads();
    // ordered compaction, 64 blocks per wave and pass
    int base = 0;
    for (int g0 = 0; g0 < G; g0 += NTH) {
        const int g = g0 + tid;
        const bool used = g < G && mask[g] != 0u;
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

template <int NS>
__global__ __launch_bounds__(FD_THREADS)
void ffn_gateup_mfma(const uint16_t* __restrict__ Wg, const uint16_t* __restrict__ Wu, int d, int G, int b,
                     const uint16_t* __restrict__ x, int T, const int32_t* __restrict__ support, int k, int shared,
                     int direct, uint16_t* __restrict__ hbuf, uint32_t* __restrict__ list_out) {
    __shared__ uint32_t mask[FD_MAXG];
    __shared__ uint16_t ulist[FD_MAXG];
    __shared__ int wcount[FD_WAVES];
    __shared__ float red[2][FD_WAVES][256];
    __shared__ int n_direct;                          // listed blocks that are handled as direct items
    // per wave: two tiles of 16 rows (8 gate, 8 up) x 128 bytes, pieces swizzled (turn_at: fragment reads without
    // bank conflicts); two pairs of k-steps are exchanged at a time, which halves the waits for LDS (1.4 us per
    // call at 16 rows)
    __shared__ __attribute__((aligned(16))) uint16_t turn[FD_WAVES][2][16 * FD_TROW];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 15, kg = lane >> 4;         // tile column / row index, k-group
    const int lr = lane >> 3, lc = lane & 7;          // as a loader: row of the half tile, 16-byte piece of the line
    // k-steps of this wave: pairs of adjacent 32-column steps = one 128-byte line per row and pair
    auto kcol = [&](int s) { return (((s >> 1) * FD_WAVES + wave) * 2 + (s & 1)) * 32; };
    const int cpb = b >> 3;                           // 8-channel chunks per block
    // row lr of the item's gate rows (its up row sits at the same offset in Wu), at piece lc of a line
    // Offsets are 32-bit element counts from the uniform bases (the host sends larger weight arrays down
    // another path): fewer address registers, 1.3 us per call at 8 and 16 rows.
    auto row_off = [&](int g, int cc) -> uint32_t { return (uint32_t)((g * b + cc * 8 + lr) * d + lc * 8); };
    // the two loads of pair p of an item: lines of the 8 gate rows, lines of the 8 up rows
    auto fetch_item = [&](bf16x8_t (&dst)[NS], uint32_t off) {
#pragma unroll
        for (int pr = 0; pr < NS / 2; ++pr) {
            const int col = (pr * FD_WAVES + wave) * 64 + lc * 8;
            const bool ok = col < d;
            const uint32_t at = off + (uint32_t)(col - lc * 8);
            dst[2 * pr] = ok ? load_frag_once(Wg + at) : zero_frag();
            dst[2 * pr + 1] = ok ? load_frag_once(Wu + at) : zero_frag();
        }
    };
    // raw lines -> fragments: a pair's two loads are written to a tile of the wave by rows and read back in
    // fragment order (lane (ln, kg): row ln, piece 4 e + kg of the line for k-step 2 pr + e)
    uint16_t* tile = turn[wave][0];
    uint16_t* tile1 = turn[wave][1];
    if (tid == 0) n_direct = 0;

    // Items are (used block, 8-channel chunk).  Which blocks are used is known only after the supports have
    // come in, a full memory round trip after the kernel started.  When the union of the supports is
    // expected to be dense (`direct`), the first item of workgroup w is therefore fixed beforehand as block
    // w / cpb, chunk w % cpb, and its weights are requested at once; should no token list that block, the
    // loads are dropped (they are in bounds whatever the supports say).  The items of all other used blocks
    // are dealt round-robin from the compacted list.
    const int nd_blocks = direct ? min(G, (int)gridDim.x / cpb) : 0;
    const bool has_direct = (int)blockIdx.x < nd_blocks * cpb;
    const int g_dir = blockIdx.x / cpb, cc_dir = blockIdx.x % cpb;

    // requested in this order: the first support entries, the direct item, this wave's slice of the token
    // rows (kept in registers for the whole kernel); loads return in order
    const int nsup = (shared || T == 1) ? k : T * k;
    const int pre = tid < nsup ? support[tid] : -1;
    bf16x8_t wb[NS], wn[NS];                          // raw lines of the current and of the next item
    if (has_direct) fetch_item(wb, row_off(g_dir, cc_dir));
    bf16x8_t xa[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int kk = kcol(s);
        xa[s] = (kk < d && ln < T) ? load_frag(x + (size_t)ln * d + kk + kg * 8) : zero_frag();
    }
    const int nblocks = build_block_list<FD_WAVES>(support, pre, T, k, shared, G, mask, ulist, wcount);
    // the list is ascending when it was compacted from the masks: its first entries are the direct blocks
    for (int i = tid; i < nblocks; i += FD_THREADS)
        if ((int)ulist[i] < nd_blocks && (i + 1 == nblocks || (int)ulist[i + 1] >= nd_blocks)) n_direct = i + 1;
    // the down kernel takes the list and the token masks from here: [0] count, [1 + i] block of slot i,
    // [1 + FD_MAXG + i] its token mask
    if (blockIdx.x == 0) {
        if (tid == 0) list_out[0] = (uint32_t)nblocks;
        for (int i = tid; i < nblocks; i += FD_THREADS) {
            const uint32_t g = ulist[i];
            list_out[1 + i] = g;
            list_out[1 + FD_MAXG + i] = mask[g];
        }
    }
    __syncthreads();
    const int nlisted = (nblocks - n_direct) * cpb;   // items dealt from the list
    const int first_listed = n_direct;
    int g_cur = 0, cc_cur = 0, j_next;
    bool v_cur;
    if (has_direct) {
        g_cur = g_dir; cc_cur = cc_dir;
        v_cur = mask[g_dir] != 0u;
        j_next = blockIdx.x;
    } else {
        const int j = blockIdx.x;
        v_cur = j < nlisted;
        if (v_cur) {
            g_cur = ulist[first_listed + j / cpb]; cc_cur = j % cpb;
            fetch_item(wb, row_off(g_cur, cc_cur));
        }
        j_next = j + (int)gridDim.x;
    }
    int buf = 0;
    bool direct_pass = has_direct;                    // a direct item that turns out unused is skipped, the listed ones follow
    while (v_cur || direct_pass) {
        direct_pass = false;
        const bool v_next = j_next < nlisted;
        int g_next = 0, cc_next = 0;
        if (v_next) {                                 // the next item's loads go out before the current one is used
            g_next = ulist[first_listed + j_next / cpb]; cc_next = j_next % cpb;
            fetch_item(wn, row_off(g_next, cc_next));
        }
        if (v_cur) {
            f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int pr = 0; pr < NS / 2; pr += 2) {
                // two pairs per exchange, each through a tile of its own: half as many waits
                bf16x8_t f[4];
                *reinterpret_cast<bf16x8_t*>(tile + turn_at(lr, lc)) = wb[2 * pr];
                *reinterpret_cast<bf16x8_t*>(tile + turn_at(8 + lr, lc)) = wb[2 * pr + 1];
                if (pr + 1 < NS / 2) {
                    *reinterpret_cast<bf16x8_t*>(tile1 + turn_at(lr, lc)) = wb[2 * pr + 2];
                    *reinterpret_cast<bf16x8_t*>(tile1 + turn_at(8 + lr, lc)) = wb[2 * pr + 3];
                }
                wave_fence_lds();
                f[0] = *reinterpret_cast<const bf16x8_t*>(tile + turn_at(ln, kg));
                f[1] = *reinterpret_cast<const bf16x8_t*>(tile + turn_at(ln, 4 + kg));
                if (pr + 1 < NS / 2) {
                    f[2] = *reinterpret_cast<const bf16x8_t*>(tile1 + turn_at(ln, kg));
                    f[3] = *reinterpret_cast<const bf16x8_t*>(tile1 + turn_at(ln, 4 + kg));
                }
                wave_fence_lds();
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[2 * pr], f[0], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[2 * pr + 1], f[1], acc, 0, 0, 0);
                if (pr + 1 < NS / 2) {
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[2 * pr + 2], f[2], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[2 * pr + 3], f[3], acc, 0, 0, 0);
                }
            }
            *reinterpret_cast<f32x4_t*>(&red[buf][wave][lane * 4]) = acc;
        }
        __syncthreads();
        // element e = lane*4 + i of a tile is (token 4*(lane/16)+i, column lane%16);
        // columns 0-7 are gate channels, 8-15 the matching up channels (32 elements further)
        if (v_cur && tid < 256) {
            const int col = (tid >> 2) & 15;
            if (col < 8) {
                float sg = 0.f, su = 0.f;
#pragma unroll
                for (int w = 0; w < FD_WAVES; ++w) { sg += red[buf][w][tid]; su += red[buf][w][tid + 32]; }
                const int tok = 4 * (tid >> 6) + (tid & 3);
                const float hv = ((mask[g_cur] >> tok) & 1u) ? sg / (1.0f + __expf(-sg)) * su : 0.f;
                hbuf[((size_t)g_cur * 16 + tok) * b + cc_cur * 8 + col] = f32_to_bf16(hv);
            }
        }
        buf ^= 1;
        g_cur = g_next; cc_cur = cc_next; v_cur = v_next;
        j_next += (int)gridDim.x;
#pragma unroll
        for (int s = 0; s < NS; ++s) wb[s] = wn[s];
    }
}

// Single-token decode (T == 1): there is nothing to share between tokens, so the first product is a
// plain matrix-vector product and the matrix cores would multiply 15 rows of padding.  A wavefront owns
// one channel of one listed block: it reads the channel's gate row and up row contiguously (1 KB per
// load instruction, all loads of both rows in flight at once), multiplies with the token by packed
// bf16 dot products, reduces over the 64 lanes and writes one hidden value.  k*b wavefronts, each with
// one memory round trip after the support entry has arrived.
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
// read-once load of 16 bytes with the non-temporal hint: here a wave's load covers whole lines (1 KB of a
// row), and the hint is worth a tenth of the streaming rate (gate/up at one row: 10.9 -> 9.9 us)
__device__ __forceinline__ uint4 load_once16(const uint16_t* p) {
    typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;
    const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(t[0], t[1], t[2], t[3]);
}
constexpr int GV_WAVES = 4;
constexpr int GV_CHUNKS = 8;                          // 512-column chunks in flight per row

__device__ __forceinline__ float dot8(const uint4& w, const uint4& v, float acc) {
    acc = __builtin_amdgcn_fdot2_f32_bf16(*reinterpret_cast<const bf16x2_t*>(&w.x), *reinterpret_cast<const bf16x2_t*>(&v.x), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(*reinterpret_cast<const bf16x2_t*>(&w.y), *reinterpret_cast<const bf16x2_t*>(&v.y), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(*reinterpret_cast<const bf16x2_t*>(&w.z), *reinterpret_cast<const bf16x2_t*>(&v.z), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(*reinterpret_cast<const bf16x2_t*>(&w.w), *reinterpret_cast<const bf16x2_t*>(&v.w), acc, false);
    return acc;
}

__global__ __launch_bounds__(GV_WAVES * 64)
void ffn_gateup_gemv(const uint16_t* __restrict__ Wg, const uint16_t* __restrict__ Wu, int d, int G, int b,
                     const uint16_t* __restrict__ x, const int32_t* __restrict__ support, int k,
                     uint16_t* __restrict__ hbuf, uint32_t* __restrict__ list_out) {
    const int lane = threadIdx.x & 63;
    const int unit = __builtin_amdgcn_readfirstlane((int)blockIdx.x * GV_WAVES + (int)(threadIdx.x >> 6));
    // the down kernel takes the list of used blocks from here (see ffn_gateup_mfma): one wavefront
    // compacts the in-range support entries, 64 at a time, in their order; every listed block is used by token 0
    if (unit == 0) {
        int base = 0;
        for (int i0 = 0; i0 < k; i0 += 64) {
            const int i = i0 + lane;
            const int g = i < k ? support[i] : -1;
            const bool used = g >= 0 && g < G;
            const unsigned long long bal = __ballot(used);
            if (used) {
                const int slot = base + __popcll(bal & ((1ull << lane) - 1ull));
                list_out[1 + slot] = (uint32_t)g;
                list_out[1 + FD_MAXG + slot] = 1u;
            }
            base += __popcll(bal);
        }
        if (lane == 0) list_out[0] = (uint32_t)base;
    }
    const int j = unit / b, c = unit - j * b;
    if (j >= k) return;
    const int g = support[j];                          // uniform over the wavefront
    if (g < 0 || g >= G) return;
    const uint16_t* wg = Wg + ((size_t)g * b + c) * d;
    const uint16_t* wu = Wu + ((size_t)g * b + c) * d;
    float sg = 0.f, su = 0.f;
    for (int e0 = 0; e0 < d; e0 += GV_CHUNKS * 512) {
        uint4 a[GV_CHUNKS], u[GV_CHUNKS], v[GV_CHUNKS];
#pragma unroll
        for (int q = 0; q < GV_CHUNKS; ++q) {
            const int e = e0 + q * 512 + lane * 8;
            const bool ok = e < d;
            a[q] = ok ? load_once16(wg + e) : make_uint4(0u, 0u, 0u, 0u);
            u[q] = ok ? load_once16(wu + e) : make_uint4(0u, 0u, 0u, 0u);
            v[q] = ok ? *reinterpret_cast<const uint4*>(x + e) : make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (int q = 0; q < GV_CHUNKS; ++q) { sg = dot8(a[q], v[q], sg); su = dot8(u[q], v[q], su); }
    }
    sg = wave_sum(sg); su = wave_sum(su);
    if (lane == 0) hbuf[(size_t)g * 16 * b + c] = f32_to_bf16(sg / (1.0f + __expf(-sg)) * su);
}

// Down projection.  16 waves per workgroup, each with one block in flight at a time: timed in alternation,
// 16 x 1 beats 16 x 2 by half a microsecond per call and 8 waves x 6 blocks by two (more waves interleave
// their load / exchange / multiply phases more finely than one wave's batches do).
constexpr int DN_WAVES = 16;
constexpr int DN_UB = 1;                              // blocks in flight per wave

__global__ __launch_bounds__(DN_WAVES * 64)
void ffn_down_mfma(const uint16_t* __restrict__ Wd, int d, int G, int b, const uint16_t* __restrict__ hbuf,
                   int T, const uint32_t* __restrict__ list_in, uint16_t* __restrict__ out) {
    // LDS sized by the number of blocks (32 KB of tiles + 6 bytes per block), not by the largest list the
    // path accepts
    extern __shared__ __attribute__((aligned(16))) unsigned char dn_lds[];
    // the waves' turning tiles (16 rows x 128 bytes each: weights arrive as whole lines, the matrix cores
    // want fragments, as in the gate/up kernel) share their memory with the partial sums, which are
    // written after the last tile has been read
    static_assert(DN_WAVES * 16 * FD_TROW * sizeof(uint16_t) >= DN_WAVES * 256 * sizeof(float), "the sums fit into the tiles' memory");
    float (*red)[256] = reinterpret_cast<float (*)[256]>(dn_lds);                       // [DN_WAVES][256]
    uint32_t* umask = reinterpret_cast<uint32_t*>(dn_lds + DN_WAVES * 16 * FD_TROW * sizeof(uint16_t));
    uint16_t* ulist = reinterpret_cast<uint16_t*>(umask + G);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint16_t* turn = reinterpret_cast<uint16_t*>(dn_lds) + wave * 16 * FD_TROW;
    const int lr = lane >> 3, lc = lane & 7;          // as a loader: row of the half tile, 16-byte piece of the line
    // the list of used blocks, written by the gate/up kernel of the same call
    // (G entries are fetched whatever the count says, so that both loads are in flight together)
    for (int i = tid; i < G; i += DN_WAVES * 64) {
        ulist[i] = (uint16_t)list_in[1 + i];
        umask[i] = list_in[1 + FD_MAXG + i];
    }
    const int nblocks = min((int)list_in[0], G);
    const int ln = lane & 15, kg = lane >> 4;
    const bool tok_ok = ln < T;                       // rows of the hidden-value operand beyond T are zero
    const int ksteps = b >> 5;                        // 32 channels per matrix instruction
    const int ntiles = (d + 15) >> 4;
    __syncthreads();
    // column tiles are dealt round-robin
    for (int tile = blockIdx.x; tile < ntiles; tile += (int)gridDim.x) {
    const int col0 = tile * 16;
    const bool row_ok = col0 + ln < d;
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
    for (int u0 = wave; u0 < nblocks; u0 += DN_WAVES * DN_UB) {
        for (int ks = 0; ks < ksteps; ks += 2) {
            bf16x8_t wa[DN_UB][2], hb[DN_UB][2];
#pragma unroll
            for (int q = 0; q < DN_UB; ++q) {
                const int u = u0 + q * DN_WAVES;
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const bool ok = u < nblocks && ks + e < ksteps;
                    const int g = u < nblocks ? ulist[u] : 0;
                    const bool tok_uses = ok && ((umask[ok ? u : 0] >> ln) & 1u);      // token ln lists block g
                    const int ch = (ks + e) * 32 + kg * 8;
                    // load e of a block: lines of rows col0 + 8 e + lr, the 64 channels of k-steps ks and ks + 1
                    const int wrow = col0 + 8 * e + lr, wch = ks * 32 + lc * 8;
                    const bool wok = u < nblocks && wch < b && wrow < d;
                    wa[q][e] = wok ? load_frag_once(Wd + ((size_t)g * d + wrow) * b + wch) : zero_frag();
                    hb[q][e] = (tok_uses && tok_ok) ? load_frag(hbuf + ((size_t)g * 16 + ln) * b + ch) : zero_frag();
                }
            }
#pragma unroll
            for (int q = 0; q < DN_UB; ++q) {
                // lines -> fragments through the wave's tile: lane (ln, kg) reads row ln, piece 4 e + kg
                *reinterpret_cast<bf16x8_t*>(turn + turn_at(lr, lc)) = wa[q][0];
                *reinterpret_cast<bf16x8_t*>(turn + turn_at(8 + lr, lc)) = wa[q][1];
                wave_fence_lds();
                const bf16x8_t f0 = *reinterpret_cast<const bf16x8_t*>(turn + turn_at(ln, kg));
                const bf16x8_t f1 = *reinterpret_cast<const bf16x8_t*>(turn + turn_at(ln, 4 + kg));
                wave_fence_lds();
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f0, hb[q][0], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f1, hb[q][1], acc, 0, 0, 0);
            }
        }
    }
    __syncthreads();                                  // every wave is done with its tile: the sums take their place
    *reinterpret_cast<f32x4_t*>(&red[wave][lane * 4]) = acc;
    __syncthreads();
    // element e = lane*4 + i is (output column 4*(lane/16)+i, token lane%16)
    if (tid < 256) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < DN_WAVES; ++w) s += red[w][tid];
        const int col = col0 + 4 * (tid >> 6) + (tid & 3), tok = (tid >> 2) & 15;
        if (tok < T && col < d) out[(size_t)tok * d + col] = f32_to_bf16(s);
    }
    __syncthreads();                                  // red[] is reused by the next tile
    }
}

// k-steps per wave of the gate/up kernel: pairs of 32-column steps dealt round-robin to the 16 waves
static int gateup_steps(int d) {
    const int pairs = (d + 63) / 64;
    return 2 * ((pairs + FD_WAVES - 1) / FD_WAVES);
}

static bool mfma_decode_ok(const FfnArgs& a) {
    return a.dtype == 1 && a.T <= 16 && a.G <= FD_MAXG && (a.d % 32) == 0 && (a.b % 32) == 0 &&
           gateup_steps(a.d) <= 16 && (long long)a.G * a.b * a.d < (1LL << 31);   // 32-bit element offsets in the gate/up kernel
}

static hipError_t run_mfma_decode(const FfnArgs& a, hipStream_t s) {
    uint16_t* hbuf = reinterpret_cast<uint16_t*>(a.scratch);
    // count, used blocks and their token masks, handed from the first kernel to the second
    uint32_t* list = reinterpret_cast<uint32_t*>(hbuf + (size_t)a.G * 16 * a.b);
    const int ns = gateup_steps(a.d);
    const int cpb = a.b / 8;
    const int union_max = a.shared ? a.k : (a.T * a.k < a.G ? a.T * a.k : a.G);
    int grid = union_max * cpb;
    if (grid > 256) grid = 256;                       // one workgroup of 16 waves per compute unit
    if (grid < 1) grid = 1;
    // a dense union is expected when the tokens list at least twice as many entries as there are blocks
    const bool guess = a.union_hint == 1 || (a.union_hint == 0 && (long)a.T * a.k >= 2L * a.G);
    const int direct = (!a.shared && a.T > 1 && guess) ? 1 : 0;
    if (a.T == 1) {
        const long units = (long)a.k * a.b;
        hipLaunchKernelGGL(ffn_gateup_gemv, dim3((unsigned)((units + GV_WAVES - 1) / GV_WAVES)), dim3(GV_WAVES * 64), 0, s,
                           (const uint16_t*)a.Wg, (const uint16_t*)a.Wu, a.d, a.G, a.b, (const uint16_t*)a.x, a.support, a.k,
                           hbuf, list);
    } else {
#define CS_GU(NSV) hipLaunchKernelGGL((ffn_gateup_mfma<NSV>), dim3(grid), dim3(FD_THREADS), 0, s, \
        (const uint16_t*)a.Wg, (const uint16_t*)a.Wu, a.d, a.G, a.b, (const uint16_t*)a.x, a.T, a.support, a.k, a.shared, direct, hbuf, list)
    if (ns <= 2) CS_GU(2); else if (ns <= 4) CS_GU(4); else if (ns <= 8) CS_GU(8); else CS_GU(16);
#undef CS_GU
    }
    int dgrid = (a.d + 15) / 16;
    if (dgrid > 256) dgrid = 256;
    const size_t dn_lds = DN_WAVES * 16 * FD_TROW * sizeof(uint16_t) + (size_t)a.G * (sizeof(uint32_t) + sizeof(uint16_t));
    hipLaunchKernelGGL(ffn_down_mfma, dim3(dgrid), dim3(DN_WAVES * 64), dn_lds, s,
                       (const uint16_t*)a.Wd, a.d, a.G, a.b, hbuf, a.T, list, (uint16_t*)a.out);
    return hipGetLastError();
}

__global__ void zero_fill_kernel(uint32_t* dst, size_t words) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += stride) dst[i] = 0u;
}

hipError_t launch_zero_fill(void* dst, size_t bytes, hipStream_t s) {
    const size_t words = bytes / 4;
    if (!words) return hipSuccess;
    const int grid = (int)((words + 255) / 256 < 2048 ? (words + 255) / 256 : 2048);
    hipLaunchKernelGGL(zero_fill_kernel, dim3(grid), dim3(256), 0, s, reinterpret_cast<uint32_t*>(dst), words);
    return hipGetLastError();
}

size_t ffn_scratch_bytes(const FfnArgs& a) {
    if (mfma_decode_ok(a)) return (size_t)a.G * 16 * a.b * sizeof(uint16_t) + (2 * FD_MAXG + 4) * sizeof(uint32_t);
    if (ffn_wide_ok(a)) return ffn_wide_scratch_bytes(a);
    if (ffn_gemm_ok(a)) return ffn_gemm_scratch_bytes(a);
    return (size_t)a.T * a.k * a.b * sizeof(float);
}

hipError_t launch_block_ffn(const FfnArgs& a, hipStream_t s) {
    if (a.T <= 0) return hipSuccess;
    if (mfma_decode_ok(a)) return run_mfma_decode(a, s);
    if (ffn_wide_ok(a)) return launch_ffn_wide(a, s);
    if (ffn_gemm_ok(a)) return launch_ffn_gemm(a, s);
    if (a.dtype == 0) return run_generic<float>(a, s);
    return run_generic<uint16_t>(a, s);
}

}  // namespace csk
