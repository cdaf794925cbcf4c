// Block-sparse gated feed-forward layer restricted to a recovered support
// (masked execution of paper Sec. 3 with the block structure of Sec. 7):
//   out[t] = sum_{g in S_t} Wd_g ( silu(Wg_g x_t) * (Wu_g x_t) ).
// Only the weight blocks named by the support are read.
#include "kernels.hpp"

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
// down kernel: a workgroup owns 16 output columns; its waves split the active
//   blocks, each multiplying the block's [16 x b] slice of Wd (one contiguous
//   run of 16 rows) with the block's hidden values, then the waves are summed.
// Hidden values travel between the two kernels as bf16 in [G][16][b] order,
// already masked by "token t uses block g".
// ---------------------------------------------------------------------------
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

// Items (gate/up) and column tiles (down) go to workgroups round-robin by default.  With CS_FD_TICKETS=1
// they are handed out by a device-wide counter instead, which pays when another stream's kernels hold some
// compute units for long (a workgroup that starts late simply takes fewer items) and costs about 1.5 us per
// kernel otherwise.
#ifndef CS_FD_TICKETS
#define CS_FD_TICKETS 0
#endif
constexpr bool FD_TICKETS = CS_FD_TICKETS != 0;
constexpr int FD_WAVES = 16;
constexpr int FD_THREADS = FD_WAVES * 64;
constexpr int FD_MAXG = 1024;

__device__ __forceinline__ bf16x8_t load_frag(const uint16_t* p) {
    return *reinterpret_cast<const bf16x8_t*>(p);
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
                     uint16_t* __restrict__ hbuf, uint32_t* __restrict__ list_out, int* __restrict__ sync) {
    __shared__ uint32_t mask[FD_MAXG];
    __shared__ uint16_t ulist[FD_MAXG];
    __shared__ int wcount[FD_WAVES];
    __shared__ float red[2][FD_WAVES][256];
    __shared__ int ticket[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 15, kg = lane >> 4;         // tile column / row index, k-group
    // k-steps of this wave: pairs of adjacent 32-column steps, so that a wave reads whole 128-byte lines
    auto kcol = [&](int s) { return (((s >> 1) * FD_WAVES + wave) * 2 + (s & 1)) * 32; };

    // the first support entries, then this wave's slice of the token rows, kept in registers (both
    // requested before the block list is built)
    const int nsup = (shared || T == 1) ? k : T * k;
    const int pre = tid < nsup ? support[tid] : -1;
    bf16x8_t xa[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int kk = kcol(s);
        xa[s] = (kk < d && ln < T) ? load_frag(x + (size_t)ln * d + kk + kg * 8) : zero_frag();
    }
    // The first item of a workgroup is its own index; the following ones are index + n gridDim.x, or, with
    // tickets, gridDim.x + the value of a device-wide counter (sync[0]), drawn two items ahead so that the
    // atomic's latency never sits on the critical path.
    int t_first = 0;
    if (FD_TICKETS && tid == 0) t_first = atomicAdd(&sync[0], 1);   // result not needed before the list is built
    const int nblocks = build_block_list<FD_WAVES>(support, pre, T, k, shared, G, mask, ulist, wcount);
    // the down kernel takes the list from here instead of building it again: [0] = count, then the blocks
    if (blockIdx.x == 0) {
        // layout: [0] count, [1 + i] = block of slot i in the low half, nothing else; [1 + FD_MAXG + i] = the
        // block's token mask (the down kernel does not fetch hidden values of tokens that do not use a block)
        if (tid == 0) list_out[0] = (uint32_t)nblocks;
        for (int i = tid; i < nblocks; i += FD_THREADS) {
            const uint32_t g = ulist[i];
            list_out[1 + i] = g;
            list_out[1 + FD_MAXG + i] = mask[g];
        }
    }
    const int cpb = b >> 3;                           // 8-channel chunks per block
    const int nitems = nblocks * cpb;
    if (tid == 0) { ticket[0] = blockIdx.x; ticket[1] = (int)gridDim.x + (FD_TICKETS ? t_first : (int)blockIdx.x); }
    __syncthreads();
    auto row_ptr = [&](int item) -> const uint16_t* {
        const int g = ulist[item / cpb], cc = item % cpb;
        const uint16_t* base = ln < 8 ? Wg : Wu;
        return base + ((size_t)g * b + cc * 8 + (ln & 7)) * d + kg * 8;
    };
    bf16x8_t wb[NS], wn[NS];
    int item = ticket[0], next = ticket[1];
    if (item < nitems) {
        const uint16_t* rp = row_ptr(item);
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int kk = kcol(s);
            wb[s] = kk < d ? load_frag(rp + kk) : zero_frag();
        }
    }
    int buf = 0, it = 0;
    while (item < nitems) {
        if (next < nitems) {
            const uint16_t* rp = row_ptr(next);
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                const int kk = kcol(s);
                wn[s] = kk < d ? load_frag(rp + kk) : zero_frag();
            }
        }
        if (tid == 0) ticket[(it & 1) + 2] = FD_TICKETS ? (int)gridDim.x + atomicAdd(&sync[0], 1)   // the item after next
                                                        : (int)blockIdx.x + (it + 2) * (int)gridDim.x;
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < NS; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[s], wb[s], acc, 0, 0, 0);
        *reinterpret_cast<f32x4_t*>(&red[buf][wave][lane * 4]) = acc;
        __syncthreads();
        // element e = lane*4 + i of a tile is (token 4*(lane/16)+i, column lane%16);
        // columns 0-7 are gate channels, 8-15 the matching up channels (32 elements further)
        if (tid < 256) {
            const int col = (tid >> 2) & 15;
            if (col < 8) {
                float sg = 0.f, su = 0.f;
#pragma unroll
                for (int w = 0; w < FD_WAVES; ++w) { sg += red[buf][w][tid]; su += red[buf][w][tid + 32]; }
                const int tok = 4 * (tid >> 6) + (tid & 3);
                const int g = ulist[item / cpb], cc = item % cpb;
                const float hv = ((mask[g] >> tok) & 1u) ? sg / (1.0f + __expf(-sg)) * su : 0.f;
                hbuf[((size_t)g * 16 + tok) * b + cc * 8 + col] = f32_to_bf16(hv);
            }
        }
        buf ^= 1;
        item = next;
        next = ticket[(it & 1) + 2];          // written before the barrier above
        ++it;
#pragma unroll
        for (int s = 0; s < NS; ++s) wb[s] = wn[s];
    }
    // the last workgroup to leave puts the counters back to zero for the next launch
    __syncthreads();
    if (FD_TICKETS && tid == 0) {
        const int gone = atomicAdd(&sync[1], 1);
        if (gone == (int)gridDim.x - 1) { sync[0] = 0; sync[1] = 0; }
    }
}

// Down projection.  8 waves per workgroup and at most 128 registers per lane, so that two
// workgroups fit on a compute unit when some units are busy with another stream's kernels.
constexpr int DN_WAVES = 8;
constexpr int DN_UB = 6;                              // blocks in flight per wave

__global__ __launch_bounds__(DN_WAVES * 64)
void ffn_down_mfma(const uint16_t* __restrict__ Wd, int d, int G, int b, const uint16_t* __restrict__ hbuf,
                   int T, const uint32_t* __restrict__ list_in, uint16_t* __restrict__ out,
                   int* __restrict__ sync) {
    __shared__ uint16_t ulist[FD_MAXG];
    __shared__ uint32_t umask[FD_MAXG];
    __shared__ float red[DN_WAVES][256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    __shared__ int ticket[2];
    int t_first = 0;
    if (FD_TICKETS && tid == 0) t_first = atomicAdd(&sync[2], 1);
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
    // column tiles are handed out like the items of the gate/up kernel: own index first, then tickets
    int tile = blockIdx.x, it = 0;
    if (tid == 0) ticket[0] = (int)gridDim.x + (FD_TICKETS ? t_first : (int)blockIdx.x);
    __syncthreads();
    while (tile < ntiles) {
    const int col0 = tile * 16;
    const bool row_ok = col0 + ln < d;
    if (tid == 0 && it > 0) ticket[it & 1] = FD_TICKETS ? (int)gridDim.x + atomicAdd(&sync[2], 1)
                                                        : (int)blockIdx.x + (it + 1) * (int)gridDim.x;
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
                    const int g = ok ? ulist[u] : 0;
                    const bool tok_uses = ok && ((umask[ok ? u : 0] >> ln) & 1u);      // token ln lists block g
                    const int ch = (ks + e) * 32 + kg * 8;
                    wa[q][e] = (ok && row_ok) ? load_frag(Wd + ((size_t)g * d + col0 + ln) * b + ch) : zero_frag();
                    hb[q][e] = (tok_uses && tok_ok) ? load_frag(hbuf + ((size_t)g * 16 + ln) * b + ch) : zero_frag();
                }
            }
#pragma unroll
            for (int q = 0; q < DN_UB; ++q)
#pragma unroll
                for (int e = 0; e < 2; ++e)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[q][e], hb[q][e], acc, 0, 0, 0);
        }
    }
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
    tile = ticket[it & 1];                            // drawn at the top of this round (or before the loop)
    ++it;
    __syncthreads();                                  // red[] and the ticket slot are reused
    }
    if (FD_TICKETS && tid == 0) {
        const int gone = atomicAdd(&sync[3], 1);
        if (gone == (int)gridDim.x - 1) { sync[2] = 0; sync[3] = 0; }
    }
}

// k-steps per wave of the gate/up kernel: pairs of 32-column steps dealt round-robin to the 16 waves
static int gateup_steps(int d) {
    const int pairs = (d + 63) / 64;
    return 2 * ((pairs + FD_WAVES - 1) / FD_WAVES);
}

static bool mfma_decode_ok(const FfnArgs& a) {
    return a.dtype == 1 && a.T <= 16 && a.G <= FD_MAXG && (a.d % 32) == 0 && (a.b % 32) == 0 &&
           gateup_steps(a.d) <= 16;
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
#define CS_GU(NSV) hipLaunchKernelGGL((ffn_gateup_mfma<NSV>), dim3(grid), dim3(FD_THREADS), 0, s, \
        (const uint16_t*)a.Wg, (const uint16_t*)a.Wu, a.d, a.G, a.b, (const uint16_t*)a.x, a.T, a.support, a.k, a.shared, hbuf, list, \
        reinterpret_cast<int*>(a.sync))
    if (ns <= 2) CS_GU(2); else if (ns <= 4) CS_GU(4); else if (ns <= 8) CS_GU(8); else CS_GU(16);
#undef CS_GU
    int dgrid = (a.d + 15) / 16;
    if (dgrid > 256) dgrid = 256;
    hipLaunchKernelGGL(ffn_down_mfma, dim3(dgrid), dim3(DN_WAVES * 64), 0, s,
                       (const uint16_t*)a.Wd, a.d, a.G, a.b, hbuf, a.T, list, (uint16_t*)a.out,
                       reinterpret_cast<int*>(a.sync));
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
    if (ffn_gemm_ok(a)) return ffn_gemm_scratch_bytes(a);
    return (size_t)a.T * a.k * a.b * sizeof(float);
}

hipError_t launch_block_ffn(const FfnArgs& a, hipStream_t s) {
    if (a.T <= 0) return hipSuccess;
    if (mfma_decode_ok(a)) return run_mfma_decode(a, s);
    if (ffn_gemm_ok(a)) return launch_ffn_gemm(a, s);
    if (a.dtype == 0) return run_generic<float>(a, s);
    return run_generic<uint16_t>(a, s);
}

}  // namespace csk
