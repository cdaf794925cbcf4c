// Head-pruned single-query attention over a key/value cache: heads are the
// structured units (paper Sec. 3, Sec. 7).  Only the kept heads' K and V are read;
// pruned heads output zeros.
//
// Split-KV streaming: a workgroup takes one (sequence, kept head, position range).
// A group of dh/8 lanes owns one cached position per step: each lane loads 16 bytes
// of the key row, the group reduces the dot product, and a running softmax
// (max, sum, weighted value accumulator) is kept per lane group.  Groups, waves and
// position ranges are merged with the usual log-sum-exp rescaling.
#include "kernels.hpp"

namespace csk {

constexpr int AT_WAVES = 4;
constexpr int AT_UNROLL = 4;

template <typename T, int DH>
__global__ __launch_bounds__(AT_WAVES * 64)
void attn_partial_kernel(const T* __restrict__ q, const T* __restrict__ K, const T* __restrict__ V,
                         int H, int L, const int32_t* __restrict__ heads, int kh,
                         int span, float* __restrict__ part) {
    constexpr int LPP = DH / 8;              // lanes per position
    constexpr int PPW = 64 / LPP;            // positions per wavefront step
    constexpr int STEP = PPW * AT_WAVES;     // positions per workgroup step
    __shared__ float sm[AT_WAVES * PPW][DH + 2];

    const int split = blockIdx.x, slot = blockIdx.y, seq = blockIdx.z;
    const int nsplit = gridDim.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % LPP, grp = lane / LPP;
    const int h = heads[seq * kh + slot];
    float* dst = part + (((size_t)seq * kh + slot) * nsplit + split) * (DH + 2);
    if (h < 0 || h >= H) {                   // invalid head index: contributes an empty partial
        for (int c = threadIdx.x; c < DH + 2; c += AT_WAVES * 64) dst[c] = (c == 0) ? -INFINITY : 0.f;
        return;
    }
    const size_t head_off = ((size_t)seq * H + h);
    const T* Kh = K + head_off * (size_t)L * DH;
    const T* Vh = V + head_off * (size_t)L * DH;
    float qf[8];
    load8(q + head_off * DH + sub * 8, qf);
    const float sc = 1.4426950408889634f / sqrtf((float)DH);     // log2(e)/sqrt(dh): scores in base 2
#pragma unroll
    for (int i = 0; i < 8; ++i) qf[i] *= sc;

    const int p_begin = split * span;
    const int p_end = min(L, p_begin + span);
    float mrun = -INFINITY, lrun = 0.f, acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;

    for (int p0 = p_begin + wave * PPW + grp; p0 < p_end + 0; p0 += STEP * AT_UNROLL) {
        float kv[AT_UNROLL][8], vv[AT_UNROLL][8];
#pragma unroll
        for (int u = 0; u < AT_UNROLL; ++u) {
            const int p = p0 + u * STEP;
            if (p < p_end) {
                load8(Kh + (size_t)p * DH + sub * 8, kv[u]);
                load8(Vh + (size_t)p * DH + sub * 8, vv[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < AT_UNROLL; ++u) {
            const int p = p0 + u * STEP;
            float s = 0.f;
            if (p < p_end) {
#pragma unroll
                for (int i = 0; i < 8; ++i) s += kv[u][i] * qf[i];
            }
            s = group_sum<LPP>(s);
            if (p < p_end) {
                const float mnew = fmaxf(mrun, s);
                const float corr = exp2f(mrun - mnew);           // mrun = -inf gives 0
                const float w = exp2f(s - mnew);
                lrun = lrun * corr + w;
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] = acc[i] * corr + w * vv[u][i];
                mrun = mnew;
            }
        }
    }
    // merge the lane groups of all waves
    const int row = wave * PPW + grp;
#pragma unroll
    for (int i = 0; i < 8; ++i) sm[row][sub * 8 + i] = acc[i];
    if (sub == 0) { sm[row][DH] = mrun; sm[row][DH + 1] = lrun; }
    __syncthreads();
    float mtot = -INFINITY;
    for (int r = 0; r < AT_WAVES * PPW; ++r) mtot = fmaxf(mtot, sm[r][DH]);
    for (int c = threadIdx.x; c < DH + 2; c += AT_WAVES * 64) {
        float v = 0.f;
        if (c < DH) {
            for (int r = 0; r < AT_WAVES * PPW; ++r) {
                const float mr = sm[r][DH];
                if (mr > -INFINITY) v += exp2f(mr - mtot) * sm[r][c];
            }
        } else if (c == DH) {
            v = mtot;
        } else {
            for (int r = 0; r < AT_WAVES * PPW; ++r) {
                const float mr = sm[r][DH];
                if (mr > -INFINITY) v += exp2f(mr - mtot) * sm[r][DH + 1];
            }
        }
        dst[c == DH ? 0 : (c < DH ? c + 2 : 1)] = v;         // layout: [max, sum, acc[DH]]
    }
}

// One thread per output element: merge the position ranges of a kept head, or
// write zeros for a pruned head.
template <typename T, int DH>
__global__ void attn_combine_kernel(const float* __restrict__ part, int H, const int32_t* __restrict__ heads,
                                    int kh, int nsplit, T* __restrict__ out) {
    const int h = blockIdx.x, seq = blockIdx.y;
    const int c = threadIdx.x;
    int slot = -1;
    for (int j = 0; j < kh; ++j)
        if (heads[seq * kh + j] == h) slot = j;
    T* o = out + ((size_t)seq * H + h) * DH;
    if (slot < 0) { store1(o + c, 0.f); return; }
    const float* pp = part + ((size_t)seq * kh + slot) * nsplit * (DH + 2);
    float mtot = -INFINITY;
    for (int s = 0; s < nsplit; ++s) mtot = fmaxf(mtot, pp[(size_t)s * (DH + 2)]);
    float num = 0.f, den = 0.f;
    for (int s = 0; s < nsplit; ++s) {
        const float* ps = pp + (size_t)s * (DH + 2);
        if (ps[0] > -INFINITY) {
            const float w = exp2f(ps[0] - mtot);
            num += w * ps[2 + c];
            den += w * ps[1];
        }
    }
    store1(o + c, den > 0.f ? num / den : 0.f);
}

static void attn_split(const AttnArgs& a, int& nsplit, int& span) {
    const long pairs = (long)a.B * a.kh;
    long want = pairs > 0 ? (2048 + pairs - 1) / pairs : 1;
    if (want < 1) want = 1;
    long sp = (a.L + want - 1) / want;
    sp = ((sp + 63) / 64) * 64;
    span = (int)sp;
    nsplit = (a.L + span - 1) / span;
}

size_t attn_scratch_bytes(const AttnArgs& a) {
    int nsplit, span;
    attn_split(a, nsplit, span);
    return (size_t)a.B * a.kh * nsplit * (a.dh + 2) * sizeof(float);
}

template <typename T, int DH>
static hipError_t run_attn(const AttnArgs& a, hipStream_t s) {
    int nsplit, span;
    attn_split(a, nsplit, span);
    float* part = reinterpret_cast<float*>(a.scratch);
    if (a.kh > 0)
        hipLaunchKernelGGL((attn_partial_kernel<T, DH>), dim3(nsplit, a.kh, a.B), dim3(AT_WAVES * 64), 0, s,
                           (const T*)a.q, (const T*)a.K, (const T*)a.V, a.H, a.L, a.heads, a.kh, span, part);
    hipLaunchKernelGGL((attn_combine_kernel<T, DH>), dim3(a.H, a.B), dim3(DH), 0, s,
                       part, a.H, a.heads, a.kh, nsplit, (T*)a.out);
    return hipGetLastError();
}

hipError_t launch_head_attn(const AttnArgs& a, hipStream_t s) {
    if (a.B <= 0) return hipSuccess;
#define CS_ATTN_CASE(TYPE, DHV) if (a.dh == DHV) return run_attn<TYPE, DHV>(a, s)
    if (a.dtype == 0) { CS_ATTN_CASE(float, 64); CS_ATTN_CASE(float, 128); CS_ATTN_CASE(float, 256); }
    else { CS_ATTN_CASE(uint16_t, 64); CS_ATTN_CASE(uint16_t, 128); CS_ATTN_CASE(uint16_t, 256); }
#undef CS_ATTN_CASE
    return hipErrorInvalidValue;
}

}  // namespace csk
