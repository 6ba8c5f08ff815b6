// Two yardstick kernels for the roofline figures: what this chip delivers when a kernel does
// nothing but the bounding operation of the path.
//   * matrix issue: every wave keeps eight independent int8 16x16x64 accumulators busy from
//     registers alone (no memory, no LDS) -- the ceiling of the int8 product;
//   * streaming: every thread reads 16 bytes and writes 8, the read/write mix of the
//     rotate-and-quantise pass (two bytes in, one byte out per element), no arithmetic.
// Both leave a checkable result so the work cannot be optimised away.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "trdq_internal.h"

namespace trdq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));

namespace {

constexpr int kIndependent = 8;   // accumulators per wave: covers the instruction's latency

__global__ __launch_bounds__(512) void peak_mfma_i8_kernel(int32_t *sink, int iters)
{
    // operands of ones: every matrix instruction adds 64 to each accumulator element
    v4i a, b;
    a.x = a.y = a.z = a.w = 0x01010101;
    b = a;
    // keep the operands opaque, or the sum is folded at compile time
    asm volatile("" : "+v"(a), "+v"(b));
    v4i acc[kIndependent];
#pragma unroll
    for (int k = 0; k < kIndependent; ++k) acc[k] = v4i{0, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < kIndependent; ++k) acc[k] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, acc[k], 0, 0, 0);
    }
    int32_t s = 0;
#pragma unroll
    for (int k = 0; k < kIndependent; ++k) s += acc[k].x + acc[k].y + acc[k].z + acc[k].w;
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__device__ __forceinline__ uint32_t hash32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// The same loop on operands of pseudo-random bytes (two A and four B fragments, so that consecutive
// instructions see different inputs).  What a matrix pipe draws depends on how many of its inputs
// toggle, and the chip sets its clock by what it draws: this is the yardstick for a product of
// quantised codes, the one above the one for the published figure.
__global__ __launch_bounds__(512) void peak_mfma_i8_data_kernel(int32_t *sink, int iters)
{
    v4i a[2], b[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int i = 0; i < 2; ++i) a[i][j] = (int)hash32(threadIdx.x * 977u + i * 31u + j * 7u + 1u);
#pragma unroll
        for (int i = 0; i < 4; ++i) b[i][j] = (int)hash32(threadIdx.x * 131u + i * 17u + j * 3u + 5u);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) asm volatile("" : "+v"(a[i]));
#pragma unroll
    for (int i = 0; i < 4; ++i) asm volatile("" : "+v"(b[i]));
    v4i acc[kIndependent];
#pragma unroll
    for (int k = 0; k < kIndependent; ++k) acc[k] = v4i{0, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < kIndependent; ++k)
            acc[k] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[k & 1], b[k >> 1], acc[k], 0, 0, 0);
    }
    int32_t s = 0;
#pragma unroll
    for (int k = 0; k < kIndependent; ++k) s += acc[k].x + acc[k].y + acc[k].z + acc[k].w;
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// NT: non-temporal accesses, which pay off once the buffers no longer fit the last-level cache
template <bool NT>
__global__ __launch_bounds__(256) void peak_stream_kernel(const v4u *__restrict__ src, v2u *__restrict__ dst,
                                                          int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
        const v4u v = NT ? __builtin_nontemporal_load(src + i) : src[i];
        // low byte of each 16-bit element, in order
        v2u o;
        o.x = (v.x & 0xff) | ((v.x >> 8) & 0xff00) | ((v.y & 0xff) << 16) | ((v.y << 8) & 0xff000000u);
        o.y = (v.z & 0xff) | ((v.z >> 8) & 0xff00) | ((v.w & 0xff) << 16) | ((v.w << 8) & 0xff000000u);
        if (NT) __builtin_nontemporal_store(o, dst + i); else dst[i] = o;
    }
}

}   // namespace

int peak_mfma_independent() { return kIndependent; }

hipError_t launch_peak_mfma_i8(int32_t *sink, int workgroups, int waves, int iters, hipStream_t st, bool random_data)
{
    if (random_data) hipLaunchKernelGGL(peak_mfma_i8_data_kernel, dim3(workgroups), dim3(64 * waves), 0, st, sink, iters);
    else hipLaunchKernelGGL(peak_mfma_i8_kernel, dim3(workgroups), dim3(64 * waves), 0, st, sink, iters);
    return hipGetLastError();
}

hipError_t launch_peak_stream(const void *src, void *dst, int64_t n_elems, hipStream_t st)
{
    const int64_t n16 = n_elems / 8;
    if (n16 == 0) return hipSuccess;
    // 16 resident workgroups of 256 threads per compute unit, each thread striding over the buffer
    int64_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    const v4u *s = static_cast<const v4u *>(src);
    v2u *d = static_cast<v2u *>(dst);
    if (3 * n_elems > (int64_t)96 << 20)
        hipLaunchKernelGGL(peak_stream_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, st, s, d, n16);
    else
        hipLaunchKernelGGL(peak_stream_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, st, s, d, n16);
    return hipGetLastError();
}

}   // namespace trdq
