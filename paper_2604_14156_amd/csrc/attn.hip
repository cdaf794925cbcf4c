// Head-pruned single-query attention over a key/value cache: heads are the
// structured units (paper Sec. 3, Sec. 7).  Only the kept heads' K and V are read;
// pruned heads output zeros.
//
// Streaming kernel: a workgroup takes one (sequence, head, position range).  A group
// of dh/8 lanes owns one cached position per step: each lane loads 16 bytes of the
// key row and of the value row, the group reduces the dot product on the lane
// crossbar, and a running softmax (max, sum, weighted value accumulator) is kept
// per lane group.  Groups and waves are merged through LDS with the usual
// log-sum-exp rescaling.  The positions of a head are split over several workgroups
// so that about eight workgroups per compute unit are in flight, and a second small
// kernel merges the partial results; a short cache is handled by one workgroup per
// head that writes the result directly.
#include "kernels.hpp"
#include "common.hpp"

namespace csk {

// tuning knobs (overridable at compile time)
#ifndef CS_AT_UNROLL
#define CS_AT_UNROLL 8
#endif
#ifndef CS_AT_WGS_WIDE
#define CS_AT_WGS_WIDE 768
#endif
#ifndef CS_AT_WGS_NARROW
#define CS_AT_WGS_NARROW 3072
#endif
constexpr int AT_UNROLL = CS_AT_UNROLL;          // key/value row pairs in flight per lane
// Two workgroup shapes.  Wide (16 waves) streams best when there is enough work for three such
// workgroups per compute unit; narrow (4 waves) cuts a small batch into more pieces.
constexpr int AT_WAVES_WIDE = 16, AT_WAVES_NARROW = 4;
constexpr int AT_WGS_WIDE = CS_AT_WGS_WIDE;      // workgroups wanted, wide shape (2 resident per compute unit)
constexpr int AT_WGS_NARROW = CS_AT_WGS_NARROW;  // workgroups wanted, narrow shape (8 resident per compute unit)
constexpr int AT_MAX_SPLIT = 32;


typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;

// eight consecutive elements of a row, kept in the form the dot product wants
template <typename T> struct Frag8;
template <> struct Frag8<float> {
    float v[8];
    __device__ __forceinline__ void load(const float* p) { load8(p, v); }
    __device__ __forceinline__ void load_once(const float* p) { load8(p, v); }
    __device__ __forceinline__ float dot(const Frag8<float>& q) const {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) s += v[i] * q.v[i];
        return s;
    }
    __device__ __forceinline__ float get(int i) const { return v[i]; }
    // acc += w * row; returns the weight actually applied
    __device__ __forceinline__ float axpy(float w, float acc[8]) const {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] += w * v[i];
        return w;
    }
};
template <> struct Frag8<uint16_t> {
    uint4 r;
    __device__ __forceinline__ void load(const uint16_t* p) { r = *reinterpret_cast<const uint4*>(p); }
    // a row of the cache is read once per call and by one workgroup: the non-temporal hint keeps it from
    // displacing anything in the caches on its way (measured on a plain streaming read: 6.3 -> 7.0 TB/s)
    __device__ __forceinline__ void load_once(const uint16_t* p) {
        typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;
        const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
        r = make_uint4(t[0], t[1], t[2], t[3]);
    }
    __device__ __forceinline__ float dot(const Frag8<uint16_t>& q) const {
        // packed bf16 dot product with fp32 accumulation: two products per instruction
        float s = 0.f;
        s = __builtin_amdgcn_fdot2_f32_bf16(*reinterpret_cast<const bf16x2_t*>(&r.x), *reinterpret_cast<const bf16x2_t*>(&q.r.x), s, false);
        s = __builtin_amdgcn_fdot2_f32_bf16(*reinterpret_cast<const bf16x2_t*>(&r.y), *reinterpret_cast<const bf16x2_t*>(&q.r.y), s, false);
        s = __builtin_amdgcn_fdot2_f32_bf16(*reinterpret_cast<const bf16x2_t*>(&r.z), *reinterpret_cast<const bf16x2_t*>(&q.r.z), s, false);
        s = __builtin_amdgcn_fdot2_f32_bf16(*reinterpret_cast<const bf16x2_t*>(&r.w), *reinterpret_cast<const bf16x2_t*>(&q.r.w), s, false);
        return s;
    }
    __device__ __forceinline__ float get(int i) const {
        const uint32_t w = i < 2 ? r.x : (i < 4 ? r.y : (i < 6 ? r.z : r.w));
        return (i & 1) ? bf16_hi(w) : bf16_lo(w);
    }
    // acc += w * row without unpacking: the weight is rounded to bf16 and paired with a zero, so
    // one packed dot product per element does the multiply-add.  Returns the rounded weight, which
    // the caller also uses in the softmax denominator so that numerator and denominator agree.
    __device__ __forceinline__ float axpy(float w, float acc[8]) const {
        const uint32_t hi = (__float_as_uint(w) + 0x8000u) & 0xFFFF0000u;    // bf16(w) in the upper half
        const uint32_t lo = hi >> 16;                                        // bf16(w) in the lower half
        const bf16x2_t wl = *reinterpret_cast<const bf16x2_t*>(&lo), wh = *reinterpret_cast<const bf16x2_t*>(&hi);
        const uint32_t rr[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bf16x2_t pr = *reinterpret_cast<const bf16x2_t*>(&rr[j]);
            acc[2 * j] = __builtin_amdgcn_fdot2_f32_bf16(pr, wl, acc[2 * j], false);
            acc[2 * j + 1] = __builtin_amdgcn_fdot2_f32_bf16(pr, wh, acc[2 * j + 1], false);
        }
        return __uint_as_float(hi);
    }
};

// Merge of the position ranges of one head for output element c: partial results are
// [max, sum, acc[DH]] per range, scores in base 2.  Two passes (the overall maximum, then the
// weighted sums), each with eight ranges' loads in flight.
template <int DH>
__device__ __forceinline__ float merge_ranges(const float* __restrict__ pp, int nsplit, int c) {
    if (nsplit <= 8) {
        // the usual case: everything is fetched in one round trip, then the same two passes on registers
        float mx[8], sm[8], ac[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float* ps = pp + (size_t)u * (DH + 2);
            const bool in = u < nsplit;
            mx[u] = in ? ps[0] : -INFINITY;
            sm[u] = in ? ps[1] : 0.f;
            ac[u] = in ? ps[2 + c] : 0.f;
        }
        float mtot = -INFINITY;
#pragma unroll
        for (int u = 0; u < 8; ++u) mtot = fmaxf(mtot, mx[u]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float w = mx[u] > -INFINITY ? exp2f(mx[u] - mtot) : 0.f;
            num += w * ac[u];
            den += w * sm[u];
        }
        return den > 0.f ? num / den : 0.f;
    }
    float mtot = -INFINITY;
    for (int s0 = 0; s0 < nsplit; s0 += 8) {
        float mx[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) mx[u] = s0 + u < nsplit ? pp[(size_t)(s0 + u) * (DH + 2)] : -INFINITY;
#pragma unroll
        for (int u = 0; u < 8; ++u) mtot = fmaxf(mtot, mx[u]);
    }
    float num = 0.f, den = 0.f;
    for (int s0 = 0; s0 < nsplit; s0 += 8) {
        float mx[8], sm[8], ac[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float* ps = pp + (size_t)(s0 + u) * (DH + 2);
            const bool in = s0 + u < nsplit;
            mx[u] = in ? ps[0] : -INFINITY;
            sm[u] = in ? ps[1] : 0.f;
            ac[u] = in ? ps[2 + c] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float w = mx[u] > -INFINITY ? exp2f(mx[u] - mtot) : 0.f;
            num += w * ac[u];
            den += w * sm[u];
        }
    }
    return den > 0.f ? num / den : 0.f;
}

template <typename T, int DH, int NW, bool FINAL>
__global__ __launch_bounds__(NW * 64)
void attn_stream_kernel(const T* __restrict__ q, const T* __restrict__ K, const T* __restrict__ V,
                        int H, int L, const int32_t* __restrict__ heads, int kh,
                        int span, int nsplit, float* __restrict__ part, T* __restrict__ out) {
    constexpr int LPP = DH / 8;              // lanes per position
    constexpr int PPW = 64 / LPP;            // positions per wavefront step
    constexpr int STEP = PPW * NW;           // positions per workgroup step
    __shared__ float sm[NW][DH + 2];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % LPP, grp = lane / LPP;
    int split, seq, slot, h;
    if (FINAL) {
        // grid (1, H, B): all heads, the pruned ones write their zeros here
        split = 0; h = blockIdx.y; seq = blockIdx.z;
        slot = -1;
        for (int j0 = 0; j0 < kh; j0 += 64) {            // one load per lane, match found by ballot
            const int j = j0 + lane;
            const int hv = j < kh ? heads[seq * kh + j] : -1;
            const unsigned long long bal = __ballot(hv == h);
            if (bal) slot = j0 + __ffsll((long long)bal) - 1;
        }
        if (slot < 0) {
            for (int c = threadIdx.x; c < DH; c += NW * 64) store1(out + ((size_t)seq * H + h) * DH + c, 0.f);
            return;
        }
    } else {
        // grid (B * kh * nsplit): kept heads only, in the order [seq][slot][range].  There are more
        // workgroups than fit on the chip at once, so the dispatcher hands the later ones to whichever
        // compute unit is free: units that get a smaller share of the memory bandwidth process fewer ranges.
        const int item = blockIdx.x;
        split = item % nsplit;
        slot = (item / nsplit) % kh;
        seq = item / (nsplit * kh);
        h = heads[seq * kh + slot];
        if (h < 0 || h >= H) return;                     // uniform; the merge kernel skips the entry too
    }
    const size_t head_off = ((size_t)seq * H + h);
    const T* Kh = K + head_off * (size_t)L * DH + sub * 8;
    const T* Vh = V + head_off * (size_t)L * DH + sub * 8;
    Frag8<T> qf;
    qf.load(q + head_off * DH + sub * 8);
    const float sc = 1.4426950408889634f / sqrtf((float)DH);     // log2(e)/sqrt(dh): scores in base 2

    const int p_begin = split * span;
    const int p_end = min(L, p_begin + span);
    float mrun = -INFINITY, lrun = 0.f, acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;

    for (int p0 = p_begin + wave * PPW + grp; p0 < p_end; p0 += STEP * AT_UNROLL) {
        Frag8<T> kv[AT_UNROLL], vv[AT_UNROLL];
#pragma unroll
        for (int u = 0; u < AT_UNROLL; ++u) {
            const int p = min(p0 + u * STEP, p_end - 1);           // clamped: loads stay in range
            kv[u].load_once(Kh + (size_t)p * DH);
            vv[u].load_once(Vh + (size_t)p * DH);
        }
        // scores of the whole batch first, then one rescale of the running state
        float sc_u[AT_UNROLL];
        float mblk = -INFINITY;
#pragma unroll
        for (int u = 0; u < AT_UNROLL; ++u) {
            const float s = group_sum<LPP>(kv[u].dot(qf)) * sc;
            sc_u[u] = (p0 + u * STEP < p_end) ? s : -INFINITY;     // u = 0 is always in range
            mblk = fmaxf(mblk, sc_u[u]);
        }
        const float mnew = fmaxf(mrun, mblk);
        const float corr = __builtin_amdgcn_exp2f(mrun - mnew);    // first batch: exp2(-inf) = 0
        mrun = mnew;
        lrun *= corr;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] *= corr;
#pragma unroll
        for (int u = 0; u < AT_UNROLL; ++u) {
            const float w = __builtin_amdgcn_exp2f(sc_u[u] - mnew);
            lrun += vv[u].axpy(w, acc);
        }
    }
    // merge the lane groups of a wave on the lane crossbar: after this every group holds the wave's state
#pragma unroll
    for (int off = LPP; off < 64; off <<= 1) {
        const float mo = __shfl_xor(mrun, off, 64), lo = __shfl_xor(lrun, off, 64);
        const float mn = fmaxf(mrun, mo);
        const float c1 = mrun > -INFINITY ? __builtin_amdgcn_exp2f(mrun - mn) : 0.f;
        const float c2 = mo > -INFINITY ? __builtin_amdgcn_exp2f(mo - mn) : 0.f;
        lrun = lrun * c1 + lo * c2;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = acc[i] * c1 + __shfl_xor(acc[i], off, 64) * c2;
        mrun = mn;
    }
    // merge the waves through LDS
    if (grp == 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) sm[wave][sub * 8 + i] = acc[i];
        if (sub == 0) { sm[wave][DH] = mrun; sm[wave][DH + 1] = lrun; }
    }
    __syncthreads();
    float mtot = -INFINITY;
#pragma unroll
    for (int r = 0; r < NW; ++r) mtot = fmaxf(mtot, sm[r][DH]);
    float wr[NW], den = 0.f;
#pragma unroll
    for (int r = 0; r < NW; ++r) {
        const float mr = sm[r][DH];
        wr[r] = mr > -INFINITY ? __builtin_amdgcn_exp2f(mr - mtot) : 0.f;
        den += wr[r] * sm[r][DH + 1];
    }
    float* dst = FINAL ? nullptr : part + (((size_t)seq * kh + slot) * nsplit + split) * (DH + 2);
    for (int c = threadIdx.x; c < DH; c += NW * 64) {
        float v = 0.f;
#pragma unroll
        for (int r = 0; r < NW; ++r) v += wr[r] * sm[r][c];
        if (FINAL) store1(out + head_off * DH + c, den > 0.f ? v / den : 0.f);
        else dst[2 + c] = v;                                     // layout: [max, sum, acc[DH]]
    }
    if (FINAL) return;
    if (threadIdx.x == 0) { dst[0] = mtot; dst[1] = den; }
}

// Merge kernel, grid (kh, B), one thread per output element: workgroup `slot` merges the position
// ranges of the head listed there and writes the zeros of those of the heads slot, slot + kh,
// slot + 2 kh, ... that are pruned (between them the kh workgroups of a sequence cover all H heads).
// A head listed twice is merged by both workgroups, with equal results.
template <typename T, int DH>
__global__ void attn_combine_kernel(const float* __restrict__ part, int H, const int32_t* __restrict__ heads,
                                    int kh, int nsplit, T* __restrict__ out) {
    const int slot = blockIdx.x, seq = blockIdx.y;
    const int c = threadIdx.x, lane = c & 63;
    const int h = heads[seq * kh + slot];
    // the loads of the merge do not depend on the head list: they are issued first
    const float* pp = part + ((size_t)seq * kh + slot) * nsplit * (DH + 2);
    const float merged = merge_ranges<DH>(pp, nsplit, c);
    for (int hp = slot; hp < H; hp += kh) {
        bool listed = false;
        for (int j0 = 0; j0 < kh; j0 += 64) {
            const int j = j0 + lane;
            listed |= __ballot(j < kh && heads[seq * kh + j] == hp) != 0ull;
        }
        if (!listed) store1(out + ((size_t)seq * H + hp) * DH + c, 0.f);
    }
    if (h < 0 || h >= H) return;
    store1(out + ((size_t)seq * H + h) * DH + c, merged);
}

// Workgroup shape, number of position ranges per head and their length.  One range (the result
// is written directly) only when the cache is short.  A range is a whole number of unrolled passes
// of a workgroup.
struct AttnShape { int nw, nsplit, span; };

static AttnShape attn_shape_for(const AttnArgs& a, int nw, long target) {
    const long pairs = (long)a.B * a.kh;
    long want = pairs > 0 ? (target + pairs - 1) / pairs : 1;
    if (want > AT_MAX_SPLIT) want = AT_MAX_SPLIT;
    long sp = (a.L + want - 1) / want;
    const long unit = (long)(64 / (a.dh / 8)) * nw * AT_UNROLL;
    sp = ((sp + unit - 1) / unit) * unit;
    AttnShape r;
    r.nw = nw;
    r.span = (int)sp;
    r.nsplit = (int)((a.L + sp - 1) / sp);
    if (r.nsplit == 1) r.span = a.L;
    return r;
}

static AttnShape attn_shape(const AttnArgs& a) {
    const AttnShape wide = attn_shape_for(a, AT_WAVES_WIDE, AT_WGS_WIDE);
    if ((long)a.B * a.kh * wide.nsplit >= 512) return wide;
    return attn_shape_for(a, AT_WAVES_NARROW, AT_WGS_NARROW);
}

size_t attn_scratch_bytes(const AttnArgs& a) {
    const AttnShape sh = attn_shape(a);
    return sh.nsplit == 1 ? 0 : (size_t)a.B * a.kh * sh.nsplit * (a.dh + 2) * sizeof(float);
}

template <typename T, int DH, int NW>
static hipError_t run_attn(const AttnArgs& a, const AttnShape& sh, hipStream_t s) {
    const int nsplit = sh.nsplit, span = sh.span;
    float* part = reinterpret_cast<float*>(a.scratch);
    if (nsplit == 1) {
        hipLaunchKernelGGL((attn_stream_kernel<T, DH, NW, true>), dim3(1, a.H, a.B), dim3(NW * 64), 0, s,
                           (const T*)a.q, (const T*)a.K, (const T*)a.V, a.H, a.L, a.heads, a.kh, span, 1, part, (T*)a.out);
    } else {
        const long nitems = (long)a.B * a.kh * nsplit;
        if (nitems > 0x7fffffffL) return hipErrorInvalidValue;
        if (nitems > 0)
            hipLaunchKernelGGL((attn_stream_kernel<T, DH, NW, false>), dim3((unsigned)nitems), dim3(NW * 64), 0, s,
                               (const T*)a.q, (const T*)a.K, (const T*)a.V, a.H, a.L, a.heads, a.kh, span, nsplit, part, (T*)a.out);
        if (a.kh > 0)
            hipLaunchKernelGGL((attn_combine_kernel<T, DH>), dim3(a.kh, a.B), dim3(DH), 0, s,
                               part, a.H, a.heads, a.kh, nsplit, (T*)a.out);
    }
    return hipGetLastError();
}

hipError_t launch_head_attn(const AttnArgs& a, hipStream_t s) {
    if (a.B <= 0) return hipSuccess;
    const AttnShape sh = attn_shape(a);
#define CS_ATTN_CASE(TYPE, DHV) if (a.dh == DHV) return sh.nw == AT_WAVES_WIDE ? run_attn<TYPE, DHV, AT_WAVES_WIDE>(a, sh, s) : run_attn<TYPE, DHV, AT_WAVES_NARROW>(a, sh, s)
    if (a.dtype == 0) { CS_ATTN_CASE(float, 64); CS_ATTN_CASE(float, 128); CS_ATTN_CASE(float, 256); }
    else { CS_ATTN_CASE(uint16_t, 64); CS_ATTN_CASE(uint16_t, 128); CS_ATTN_CASE(uint16_t, 256); }
#undef CS_ATTN_CASE
    return hipErrorInvalidValue;
}

}  // namespace csk
