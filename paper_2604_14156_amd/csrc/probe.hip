// Diagnostic: a plain streaming read.  The bandwidth-bound calls of the library (block-sparse FFN at
// decode, head-pruned attention; the paper's Sec. 14 names memory bandwidth and KV-cache traffic as what
// decides latency) are reported against the published peak of the device and, beside it, against what
// this kernel reaches on the same device in the same run.
#include "kernels.hpp"
#include "common.hpp"

namespace csk {

constexpr int PR_THREADS = 1024;
constexpr int PR_UNROLL = 8;          // 16-byte loads in flight per lane
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;

__global__ __launch_bounds__(PR_THREADS)
void stream_read_kernel(const uint4* __restrict__ src, size_t n16, uint32_t* __restrict__ checksum) {
    // a workgroup takes contiguous pieces of PR_THREADS * PR_UNROLL 16-byte words (128 KB) in turn; within
    // a piece a wavefront's load instruction covers 1 KB of consecutive addresses
    constexpr size_t PIECE = (size_t)PR_THREADS * PR_UNROLL;
    uint32_t acc = 0u;
    for (size_t base = (size_t)blockIdx.x * PIECE; base < n16; base += (size_t)gridDim.x * PIECE) {
        uint4 v[PR_UNROLL];
#pragma unroll
        for (int u = 0; u < PR_UNROLL; ++u) {
            const size_t i = base + (size_t)u * PR_THREADS + threadIdx.x;
            // read once: the non-temporal hint is worth about a tenth of the rate on this device
            if (i < n16) {
                const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(src) + i);
                v[u] = make_uint4(t[0], t[1], t[2], t[3]);
            } else {
                v[u] = make_uint4(0u, 0u, 0u, 0u);
            }
        }
#pragma unroll
        for (int u = 0; u < PR_UNROLL; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    // one atomic per workgroup keeps the loads from being optimised away and makes the result checkable
    // (atomics on one address are serialised by the memory system: a few thousand per launch are free,
    // one per wavefront of a large grid is not)
    __shared__ uint32_t part[PR_THREADS / 64];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc ^= __shfl_xor(acc, off, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t v = 0u;
#pragma unroll
        for (int w = 0; w < PR_THREADS / 64; ++w) v ^= part[w];
        if (v != 0u) atomicXor(checksum, v);
    }
}

hipError_t launch_stream_read(const void* src, size_t bytes, uint32_t* checksum, hipStream_t s) {
    const size_t n16 = bytes / 16;
    if (!n16) return hipSuccess;
    size_t blocks = (n16 + (size_t)PR_THREADS * PR_UNROLL - 1) / ((size_t)PR_THREADS * PR_UNROLL);
    if (blocks > 1024) blocks = 1024;                 // 4 workgroups per compute unit, grid-stride beyond
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(PR_THREADS), 0, s,
                       reinterpret_cast<const uint4*>(src), n16, checksum);
    return hipGetLastError();
}

}  // namespace csk
