// Calibration-side reductions: what Eq. 5 (the smoothing diagonal) and the zigzag permutation of
// Sec. 3.2 are built from.
//   channel_absmax:     mag[k]  = max_i |(X . diag)[i, k]|, optionally after the block rotation
//                                 (max_i |((X . diag) . R)[i, k]|, R orthonormal)
//   weight_row_absmax:  wmax[k] = max_n |W[k, n]|
//   smooth_diag:        d[k]    = wmax[k]^(1 - alpha) / xmax[k]^alpha   (the reciprocal of Delta_k of
//                                 Eq. 5, because this library multiplies activations by d);
//                                 a channel whose xmax or wmax is zero gets d = 1
// Offline work (once per time-step group); plain streaming kernels.
#include "device_utils.h"
#include "trdq_internal.h"

namespace trdq {

namespace {

__global__ void fill_zero_kernel(float *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

// in-lane H_8 over 8 values (three add stages)
__device__ __forceinline__ void cal_h8(float (&v)[8])
{
    const float b0 = v[0] + v[1], b1 = v[0] - v[1], b2 = v[2] + v[3], b3 = v[2] - v[3];
    const float b4 = v[4] + v[5], b5 = v[4] - v[5], b6 = v[6] + v[7], b7 = v[6] - v[7];
    const float a0 = b0 + b2, a2 = b0 - b2, a1 = b1 + b3, a3 = b1 - b3;
    const float a4 = b4 + b6, a6 = b4 - b6, a5 = b5 + b7, a7 = b5 - b7;
    v[0] = a0 + a4; v[4] = a0 - a4;
    v[1] = a1 + a5; v[5] = a1 - a5;
    v[2] = a2 + a6; v[6] = a2 - a6;
    v[3] = a3 + a7; v[7] = a3 - a7;
}

// A wave works on one block of 128 channels and walks token groups of 16 with a stride, keeping
// a running maximum per channel in 32 registers per lane: lane (g, r) holds token r and, with
// ROTATE, output chunks 4g .. 4g+3 of the block (8 channels each); without, input chunks 4s + g,
// s = 0..3.  At the end the 16 tokens of a lane row are reduced with row moves and one lane per
// row issues the atomic maxima (non-negative floats compare like their bit patterns).  The
// rotation is the fp32 form used by rotate_quant_rpr (H_8 in the lane, H_16 as an exact product
// with a +-1 matrix on the matrix cores).
template <bool ROTATE>
__global__ __launch_bounds__(256) void channel_absmax_kernel(
    const uint16_t *__restrict__ X, int64_t M, int nb, int64_t ldx,
    const float *__restrict__ diag, float *__restrict__ mag)
{
    const int lane = threadIdx.x & 63;
    const int g = lane >> 4, r = lane & 15;
    const int64_t groups = (M + 15) / 16;
    // waves of the grid: wave w of the launch works on block w % nb, token groups (w / nb), + stride
    const int64_t gw = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    const int b = (int)(gw % nb);
    const int64_t first = gw / nb, stride = nwaves / nb;      // launcher makes nwaves a multiple of nb
    if (stride == 0 || first >= stride) return;

    float hn[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) hn[s] = (__builtin_popcount(r & (4 * s + g)) & 1) ? -1.0f : 1.0f;

    float mx[4][8];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int j = 0; j < 8; ++j) mx[q][j] = 0.0f;

    for (int64_t tg = first; tg < groups; tg += stride) {
        int64_t token = tg * 16 + r;
        if (token >= M) token = M - 1;               // a repeated token does not change a maximum
        float w[4][8];
        const uint16_t *src = X + token * ldx + b * kBlock + g * 8;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const uint4 qv = *reinterpret_cast<const uint4 *>(src + s * 32);
            float4 d0 = make_float4(1.f, 1.f, 1.f, 1.f), d1 = d0;
            if (diag) {
                const float *dp = diag + b * kBlock + (4 * s + g) * 8;
                d0 = *reinterpret_cast<const float4 *>(dp);
                d1 = *reinterpret_cast<const float4 *>(dp + 4);
            }
            w[s][0] = bf16_lo(qv.x) * d0.x; w[s][1] = bf16_hi(qv.x) * d0.y;
            w[s][2] = bf16_lo(qv.y) * d0.z; w[s][3] = bf16_hi(qv.y) * d0.w;
            w[s][4] = bf16_lo(qv.z) * d1.x; w[s][5] = bf16_hi(qv.z) * d1.y;
            w[s][6] = bf16_lo(qv.w) * d1.z; w[s][7] = bf16_hi(qv.w) * d1.w;
            if (ROTATE) cal_h8(w[s]);
        }
        if (ROTATE) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                v4f acc = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(hn[s], w[s][j], acc, 0, 0, 0);
#pragma unroll
                for (int q = 0; q < 4; ++q) mx[q][j] = fmaxf(mx[q][j], fabsf(acc[q]));
            }
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int j = 0; j < 8; ++j) mx[s][j] = fmaxf(mx[s][j], fabsf(w[s][j]));
        }
    }

    // chunk index of mx[q]: rotated -> output chunk 4g + q; raw -> input chunk 4q + g
    const float norm = ROTATE ? 0.08838834764831845f : 1.0f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int chunk = ROTATE ? 4 * g + q : 4 * q + g;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float m = row16_max(mx[q][j]) * norm;
            if (r == 0)
                atomicMax(reinterpret_cast<unsigned int *>(mag + b * kBlock + chunk * 8 + j), __float_as_uint(m));
        }
    }
}

__global__ __launch_bounds__(256) void weight_row_absmax_kernel(const float *__restrict__ W, int K, int N,
                                                                float *__restrict__ wmax)
{
    __shared__ float part[4];
    const int k = blockIdx.x;
    float m = 0.0f;
    for (int n = threadIdx.x; n < N; n += blockDim.x) m = fmaxf(m, fabsf(W[(size_t)k * N + n]));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) wmax[k] = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
}

__global__ void smooth_diag_kernel(const float *__restrict__ xmax, const float *__restrict__ wmax, int K,
                                   float alpha, float *__restrict__ d)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    const float x = xmax[k], w = wmax[k];
    d[k] = (x > 0.0f && w > 0.0f) ? powf(w, 1.0f - alpha) / powf(x, alpha) : 1.0f;
}

}  // namespace

hipError_t launch_channel_absmax(const uint16_t *X, int64_t M, int K, int64_t ldx, const float *diag,
                                 bool rotate, float *mag, hipStream_t st)
{
    hipLaunchKernelGGL(fill_zero_kernel, dim3((K + 255) / 256), dim3(256), 0, st, mag, K);
    if (M == 0) return hipGetLastError();
    const int nb = K / kBlock;
    const int64_t groups = (M + 15) / 16;
    // waves = nb x (token-group lanes): about 8 waves per SIMD over the chip, at least one per block
    int64_t per_block = (256 * 4 * 8) / nb;
    if (per_block > groups) per_block = groups;
    if (per_block < 1) per_block = 1;
    int64_t waves = per_block * nb;
    waves = (waves + 3) / 4 * 4;                     // whole workgroups of four waves ...
    while (waves % nb != 0) waves += 4;              // ... and a multiple of nb
    const unsigned grid = (unsigned)(waves / 4);
    if (rotate)
        hipLaunchKernelGGL(channel_absmax_kernel<true>, dim3(grid), dim3(256), 0, st, X, M, nb, ldx, diag, mag);
    else
        hipLaunchKernelGGL(channel_absmax_kernel<false>, dim3(grid), dim3(256), 0, st, X, M, nb, ldx, diag, mag);
    return hipGetLastError();
}

hipError_t launch_weight_row_absmax(const float *W, int K, int N, float *wmax, hipStream_t st)
{
    hipLaunchKernelGGL(weight_row_absmax_kernel, dim3(K), dim3(256), 0, st, W, K, N, wmax);
    return hipGetLastError();
}

hipError_t launch_smooth_diag(const float *xmax, const float *wmax, int K, float alpha, float *d, hipStream_t st)
{
    hipLaunchKernelGGL(smooth_diag_kernel, dim3((K + 255) / 256), dim3(256), 0, st, xmax, wmax, K, alpha, d);
    return hipGetLastError();
}

}  // namespace trdq
