// Attention sharing (Sec. 3.3): the cosine similarity of Eq. 11 between the attention outputs of the
// conditional and the unconditional pass, one value per segment (a transformer block's output, a
// head, ...).  A streaming reduction: 4 bytes read per element pair, nothing else.
//   cos[s] = A_s . B_s / (|A_s| |B_s|);   0 where either vector is all zero.
// A product of two bf16 values is exact in fp32; a lane adds 64 of them in fp32 (relative error
// below 64 * 2^-24 of the sum of magnitudes), then carries on in fp64: per-wave sums are merged
// with fp64 atomic adds into three accumulators per segment, which a second kernel turns into the
// cosine.  The order of the atomic adds varies from run to run; in fp64 that moves the result
// by parts in 10^16.
#include "device_utils.h"
#include <map>
#include <mutex>

#include "trdq_internal.h"

namespace trdq {

namespace {

__global__ void fill_zero_f64_kernel(double *p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0;
}

__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// grid: (chunks per segment, segments).  A workgroup walks its share of the segment in steps of
// 256 lanes x 8 elements; the tail (seg_len % 8) is taken element by element by the last chunk.
__global__ __launch_bounds__(256) void cosine_accumulate_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ B, int64_t seg_len, int64_t stride_a,
    int64_t stride_b, double *__restrict__ acc)
{
    __shared__ double part[4][3];
    const int s = blockIdx.y;
    const uint16_t *a = A + (int64_t)s * stride_a;
    const uint16_t *b = B + (int64_t)s * stride_b;
    const int64_t vec = seg_len / 8;                                  // whole 16-byte pieces
    double dd = 0.0, da = 0.0, db = 0.0;
    float fd = 0.0f, fa = 0.0f, fb = 0.0f;
    int run = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < vec; i += (int64_t)gridDim.x * blockDim.x) {
        const uint4 x = *reinterpret_cast<const uint4 *>(a + i * 8);
        const uint4 y = *reinterpret_cast<const uint4 *>(b + i * 8);
        const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float x0 = bf16_lo(xs[j]), x1 = bf16_hi(xs[j]), y0 = bf16_lo(ys[j]), y1 = bf16_hi(ys[j]);
            fd = __builtin_fmaf(x0, y0, fd); fd = __builtin_fmaf(x1, y1, fd);
            fa = __builtin_fmaf(x0, x0, fa); fa = __builtin_fmaf(x1, x1, fa);
            fb = __builtin_fmaf(y0, y0, fb); fb = __builtin_fmaf(y1, y1, fb);
        }
        if (++run == 8) {                                             // 64 products per fp32 sum
            dd += (double)fd; da += (double)fa; db += (double)fb;
            fd = fa = fb = 0.0f;
            run = 0;
        }
    }
    dd += (double)fd; da += (double)fa; db += (double)fb;
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x < (unsigned)(seg_len - vec * 8)) {
        const float x0 = bf16_lo(a[vec * 8 + threadIdx.x]), y0 = bf16_lo(b[vec * 8 + threadIdx.x]);
        dd += (double)x0 * (double)y0; da += (double)x0 * (double)x0; db += (double)y0 * (double)y0;
    }
    dd = wave_sum(dd); da = wave_sum(da); db = wave_sum(db);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { part[wave][0] = dd; part[wave][1] = da; part[wave][2] = db; }
    __syncthreads();
    if (threadIdx.x < 3) {
        const double t = part[0][threadIdx.x] + part[1][threadIdx.x] + part[2][threadIdx.x] + part[3][threadIdx.x];
        atomicAdd(acc + (int64_t)s * 3 + threadIdx.x, t);
    }
}

__global__ void cosine_finish_kernel(const double *__restrict__ acc, int n_seg, float *__restrict__ out)
{
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n_seg) return;
    const double d = acc[s * 3], na = acc[s * 3 + 1], nb = acc[s * 3 + 2];
    out[s] = (na > 0.0 && nb > 0.0) ? (float)(d / (sqrt(na) * sqrt(nb))) : 0.0f;
}

// Accumulators of the entry point that allocates nothing: three float64 sums per segment, held by
// every GPU the library runs on until the process ends (96 KB).  Host code never passes this name to
// a kernel or a runtime call: it asks for the device's address of the array once per device
// (static_scratch below) and uses that pointer.
__device__ __align__(256) double scratch[3 * kCosineStaticMaxSeg];

}  // namespace

hipError_t cosine_static_scratch(double **out)
{
    static std::mutex mu;
    static std::map<int, double *> per_device;      // each GPU holds its own copy at its own address
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    auto it = per_device.find(dev);
    if (it == per_device.end()) {
        double *ptr = nullptr;
        if (hipError_t e = hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch)); e != hipSuccess)
            return e;
        if (!ptr) return hipErrorInvalidSymbol;
        it = per_device.emplace(dev, ptr).first;
    }
    *out = it->second;
    return hipSuccess;
}

hipError_t launch_cosine_similarity(const uint16_t *A, const uint16_t *B, int n_seg, int64_t seg_len,
                                    int64_t stride_a, int64_t stride_b, double *acc_ws, float *out, hipStream_t st)
{
    const int64_t n_acc = (int64_t)n_seg * 3;
    hipLaunchKernelGGL(fill_zero_f64_kernel, dim3((unsigned)((n_acc + 255) / 256)), dim3(256), 0, st, acc_ws, n_acc);
    // about eight workgroups per compute unit over all segments, each with at least a few steps
    const int64_t vec = seg_len / 8;
    int64_t chunks = (256 * 8 + n_seg - 1) / n_seg;
    const int64_t most = (vec + 256 * 4 - 1) / (256 * 4);
    if (chunks > most) chunks = most;
    if (chunks < 1) chunks = 1;
    hipLaunchKernelGGL(cosine_accumulate_kernel, dim3((unsigned)chunks, (unsigned)n_seg), dim3(256), 0, st,
                       A, B, seg_len, stride_a, stride_b, acc_ws);
    hipLaunchKernelGGL(cosine_finish_kernel, dim3((unsigned)((n_seg + 255) / 256)), dim3(256), 0, st, acc_ws, n_seg, out);
    return hipGetLastError();
}

}  // namespace trdq
