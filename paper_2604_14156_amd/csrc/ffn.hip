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
    return (size_t)a.T * a.k * a.b * sizeof(float);
}

hipError_t launch_block_ffn(const FfnArgs& a, hipStream_t s) {
    if (a.T <= 0) return hipSuccess;
    if (a.dtype == 0) return run_generic<float>(a, s);
    return run_generic<uint16_t>(a, s);
}

}  // namespace csk
