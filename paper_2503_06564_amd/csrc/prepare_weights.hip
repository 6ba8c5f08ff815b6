// prepare_weights: H_t(W) = R^T . (Delta_t^-1 . W) of Eq. 10 and the symmetric weight
// quantiser (per output channel for int8, per 128-row group and output channel for int4).
// Offline, once per time-step group; two streaming kernels through a float32 scratch matrix.
#include "device_utils.h"
#include "trdq_internal.h"

namespace trdq {

namespace {

constexpr int kCols = 64;          // output channels per workgroup
constexpr int kPrepThreads = 256;

// Kernel 1: one workgroup rotates one 128-row block of 64 columns.
//   Wrot[b*128 + j, n] = sum_k H[k][j] * W[row(b*128 + k), n] / d[b*128 + k]      (unnormalised H)
//   amax[b, n]         = max_j |Wrot[b*128 + j, n]|
// row(k) = k, or perm[k] (clamped to the matrix) when a permutation is given: the P^T factor of
// Eq. 9 in front of the second rotation.
__global__ __launch_bounds__(kPrepThreads) void prepare_rotate_kernel(
    const float *__restrict__ W, int K, int N, const float *__restrict__ diag,
    const int32_t *__restrict__ perm, float *__restrict__ Wrot, float *__restrict__ amax)
{
    __shared__ float tile[kBlock][kCols + 1];
    __shared__ float part[4][kCols];
    const int b = blockIdx.y;
    const int n0 = blockIdx.x * kCols;
    const int c = threadIdx.x % kCols;
    const int q = threadIdx.x / kCols;     // 0..3
    const int n = n0 + c;
    const bool col_ok = n < N;

    for (int k = q; k < kBlock; k += 4) {
        float w = 0.0f;
        if (col_ok) {
            int row = b * kBlock + k;
            if (perm) {
                row = perm[row];
                row = row < 0 ? 0 : (row >= K ? K - 1 : row);
            }
            w = W[(size_t)row * N + n];
            if (diag) w = w / diag[b * kBlock + k];
        }
        tile[k][c] = w;
    }
    __syncthreads();
    // 7 butterfly stages down the rows; 64 pairs per column per stage, 16 per thread
    for (int h = 1; h < kBlock; h <<= 1) {
        for (int pr = q; pr < kBlock / 2; pr += 4) {
            const int lo = ((pr / h) * 2 * h) + (pr % h);
            const float a = tile[lo][c], bb = tile[lo + h][c];
            tile[lo][c] = a + bb;
            tile[lo + h][c] = a - bb;
        }
        __syncthreads();
    }
    float m = 0.0f;
    for (int k = q; k < kBlock; k += 4) {
        const float w = tile[k][c];
        m = fmaxf(m, fabsf(w));
        if (col_ok) Wrot[(size_t)(b * kBlock + k) * N + n] = w;
    }
    part[q][c] = m;
    __syncthreads();
    if (q == 0 && col_ok)
        amax[(size_t)b * N + n] = fmaxf(fmaxf(part[0][c], part[1][c]), fmaxf(part[2][c], part[3][c]));
}

// Kernel 1 with a dense rotation block in place of the butterflies (H_t(W) = R^T (Delta^-1 W) with
// the blocks of the BlockDiag equation as arbitrary orthogonal matrices):
//   Wrot[b*128 + j, n] = sum_k R_b[k][j] * W[b*128 + k, n] / d[b*128 + k]
// Wave q of the workgroup produces rows j = 32 q .. 32 q + 31 of 64 columns; the row of R_b it
// needs at step k is the same for all its lanes (scalar loads), the column of W comes from LDS.
__global__ __launch_bounds__(kPrepThreads) void prepare_rotate_dense_kernel(
    const float *__restrict__ W, int K, int N, const float *__restrict__ diag, const int32_t *__restrict__ perm,
    const float *__restrict__ R, float *__restrict__ Wrot, float *__restrict__ amax)
{
    __shared__ float tile[kBlock][kCols + 1];
    __shared__ float part[4][kCols];
    const int b = blockIdx.y;
    const int n0 = blockIdx.x * kCols;
    const int c = threadIdx.x % kCols;
    const int q = __builtin_amdgcn_readfirstlane(threadIdx.x / kCols);     // 0..3, one wave each
    const int n = n0 + c;
    const bool col_ok = n < N;
    for (int k = q; k < kBlock; k += 4) {
        float w = 0.0f;
        if (col_ok) {
            int row = b * kBlock + k;
            if (perm) {                                  // the P^T factor in front of a second rotation
                row = perm[row];
                row = row < 0 ? 0 : (row >= K ? K - 1 : row);
            }
            w = W[(size_t)row * N + n];
            if (diag) w = w / diag[b * kBlock + k];
        }
        tile[k][c] = w;
    }
    __syncthreads();
    float acc[32];
#pragma unroll
    for (int jj = 0; jj < 32; ++jj) acc[jj] = 0.0f;
    const float *Rb = R + (size_t)b * kBlock * kBlock + 32 * q;
    for (int k = 0; k < kBlock; ++k) {
        const float w = tile[k][c];
#pragma unroll
        for (int jj = 0; jj < 32; ++jj) acc[jj] = __builtin_fmaf(Rb[k * kBlock + jj], w, acc[jj]);
    }
    float m = 0.0f;
#pragma unroll
    for (int jj = 0; jj < 32; ++jj) {
        m = fmaxf(m, fabsf(acc[jj]));
        if (col_ok) Wrot[(size_t)(b * kBlock + 32 * q + jj) * N + n] = acc[jj];
    }
    part[q][c] = m;
    __syncthreads();
    if (q == 0 && col_ok)
        amax[(size_t)b * N + n] = fmaxf(fmaxf(part[0][c], part[1][c]), fmaxf(part[2][c], part[3][c]));
}

// Kernel 2: quantise and transpose one 128-row block of 64 columns into the K-contiguous
// layouts the product kernels read (see Weights in trdq_internal.h).
//   wbits 8: scale[n]    = max_b amax[b, n] * norm / 127   (qmax = 31 in the same layout: 6-bit codes)
//   wbits 4: scale[b, n] = amax[b, n]       * norm / 7
// norm undoes the unnormalised butterflies: 1/sqrt(128) after one rotation, 1/128 after two.
//   code = rint(Wrot * qmax / amax)   (ties to even; amax == 0 -> 0)
template <int WBITS>
__global__ __launch_bounds__(kPrepThreads) void prepare_quant_kernel(
    const float *__restrict__ Wrot, const float *__restrict__ amax, int K, int N, float norm, float qmax,
    void *__restrict__ codes, float *__restrict__ scales)
{
    __shared__ int8_t q8[kCols][kBlock + 16];
    __shared__ float inv_s[kCols];
    const int nb = K / kBlock;
    const int b = blockIdx.y;
    const int n0 = blockIdx.x * kCols;

    if (threadIdx.x < kCols) {
        const int n = n0 + threadIdx.x;
        float a = 0.0f;
        if (n < N) {
            if (WBITS == 8) {
                for (int bb = 0; bb < nb; ++bb) a = fmaxf(a, amax[(size_t)bb * N + n]);
                if (b == 0) scales[n] = a * (norm / qmax);
            } else {
                a = amax[(size_t)b * N + n];
                scales[(size_t)b * N + n] = a * (norm / qmax);
            }
        }
        inv_s[threadIdx.x] = a > 0.0f ? qmax / a : 0.0f;
    }
    __syncthreads();
    const int c = threadIdx.x % kCols;
    const int q = threadIdx.x / kCols;
    const int n = n0 + c;
    for (int k = q; k < kBlock; k += 4) {
        float w = n < N ? Wrot[(size_t)(b * kBlock + k) * N + n] : 0.0f;
        q8[c][k] = (int8_t)(quant_bits(w, inv_s[c]) & 0xFF);
    }
    __syncthreads();
    if (WBITS == 8) {
        // 64 columns x 128 bytes -> 16-byte chunks, K contiguous
        int8_t *out = static_cast<int8_t *>(codes);
        for (int ch = threadIdx.x; ch < kCols * (kBlock / 16); ch += kPrepThreads) {
            const int cc = ch / (kBlock / 16), kk = (ch % (kBlock / 16)) * 16;
            if (n0 + cc < N)
                *reinterpret_cast<uint4 *>(out + (size_t)(n0 + cc) * K + b * kBlock + kk) =
                    *reinterpret_cast<const uint4 *>(&q8[cc][kk]);
        }
    } else {
        // 8 consecutive k -> 4 bytes: byte j = code(k0+j) & 0xF | (code(k0+4+j) & 0xF) << 4
        uint8_t *out = static_cast<uint8_t *>(codes);
        for (int u = threadIdx.x; u < kCols * (kBlock / 8); u += kPrepThreads) {
            const int cc = u / (kBlock / 8), k0 = (u % (kBlock / 8)) * 8;
            if (n0 + cc < N) {
                uint32_t word = 0;
                for (int j = 0; j < 4; ++j) {
                    const uint32_t lo = (uint8_t)q8[cc][k0 + j] & 0xFu;
                    const uint32_t hi = (uint8_t)q8[cc][k0 + 4 + j] & 0xFu;
                    word |= (lo | (hi << 4)) << (8 * j);
                }
                *reinterpret_cast<uint32_t *>(out + (size_t)(n0 + cc) * (K / 2) + (b * kBlock + k0) / 2) = word;
            }
        }
    }
}

// Asymmetric weights (Eq. 1-3 on H_t(W), one range per output channel).  Kernel A: lo[n] = min(min_k Wrot[k,n], 0),
// hi[n] = max(max_k Wrot[k,n], 0) over the whole column, one thread per channel.
__global__ __launch_bounds__(kPrepThreads) void column_minmax_kernel(const float *__restrict__ Wrot, int K, int N,
                                                                      float *__restrict__ lo, float *__restrict__ hi)
{
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    float a = 0.0f, b = 0.0f;
    for (int k = 0; k < K; ++k) {
        const float w = Wrot[(size_t)k * N + n];
        a = fminf(a, w);
        b = fmaxf(b, w);
    }
    lo[n] = a;
    hi[n] = b;
}

// Kernel B: s[n] = (hi - lo) * norm / 255, z[n] = -rint(lo * 255 / (hi - lo)), code = clamp(rint(w * 255 / (hi - lo)) + z,
// 0, 255), stored as code - 128 (the operand type of the int8 matrix instruction) in the [N, K] layout; zcw[n] = 128 - z,
// so that q - z = stored + zcw.  The integer offset rides in the rounding constant of one fused multiply-add.
__global__ __launch_bounds__(kPrepThreads) void prepare_quant_asym_kernel(
    const float *__restrict__ Wrot, const float *__restrict__ lo, const float *__restrict__ hi, int K, int N, float norm,
    int8_t *__restrict__ codes, float *__restrict__ scales, int32_t *__restrict__ zcw)
{
    __shared__ int8_t q8[kCols][kBlock + 16];
    __shared__ float inv_s[kCols], magic_s[kCols];
    const int b = blockIdx.y;
    const int n0 = blockIdx.x * kCols;
    if (threadIdx.x < kCols) {
        const int n = n0 + threadIdx.x;
        float inv = 0.0f, z = 0.0f;
        if (n < N) {
            const float range = hi[n] - lo[n];
            inv = range > 0.0f ? 255.0f / range : 0.0f;
            z = -rintf(lo[n] * inv);
            if (b == 0) {
                scales[n] = range * (norm / 255.0f);
                zcw[n] = 128 - (int)z;
            }
        }
        inv_s[threadIdx.x] = inv;
        magic_s[threadIdx.x] = kRoundMagic + (z - 128.0f);
    }
    __syncthreads();
    const int c = threadIdx.x % kCols;
    const int q = threadIdx.x / kCols;
    const int n = n0 + c;
    for (int k = q; k < kBlock; k += 4) {
        const float w = n < N ? Wrot[(size_t)(b * kBlock + k) * N + n] : 0.0f;
        const float t = __builtin_fmaf(w, inv_s[c], magic_s[c]);
        q8[c][k] = (int8_t)(__float_as_uint(__builtin_amdgcn_fmed3f(t, kRoundMagic - 128.0f, kRoundMagic + 127.0f)) & 0xFF);
    }
    __syncthreads();
    for (int ch = threadIdx.x; ch < kCols * (kBlock / 16); ch += kPrepThreads) {
        const int cc = ch / (kBlock / 16), kk = (ch % (kBlock / 16)) * 16;
        if (n0 + cc < N)
            *reinterpret_cast<uint4 *>(codes + (size_t)(n0 + cc) * K + b * kBlock + kk) =
                *reinterpret_cast<const uint4 *>(&q8[cc][kk]);
    }
}

// colsum[n] = sum_k codes[n][k]: one wave per output channel (the zero-point term of asymmetric
// activations needs it in the product's epilogue)
__global__ __launch_bounds__(64) void weight_colsum_kernel(const int8_t *__restrict__ codes, int K, int N,
                                                           int32_t *__restrict__ colsum)
{
    const int n = blockIdx.x;
    const int8_t *row = codes + (size_t)n * K;
    int t = 0;
    for (int k = threadIdx.x * 16; k < K; k += 64 * 16) {
        const int4 v = *reinterpret_cast<const int4 *>(row + k);
        const int wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int u = 0; u < 4; ++u)
            t += (int)(int8_t)(wv[u] & 0xFF) + (int)(int8_t)((wv[u] >> 8) & 0xFF) +
                 (int)(int8_t)((wv[u] >> 16) & 0xFF) + (wv[u] >> 24);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o);
    if (threadIdx.x == 0) colsum[n] = t;
}

}  // namespace

hipError_t launch_prepare_quant_asym(const float *Wrot, float *lohi, int K, int N, float norm, void *codes, float *scales,
                                     int32_t *zcw, hipStream_t st)
{
    float *lo = lohi, *hi = lohi + N;
    hipLaunchKernelGGL(column_minmax_kernel, dim3((N + kPrepThreads - 1) / kPrepThreads), dim3(kPrepThreads), 0, st, Wrot, K, N,
                       lo, hi);
    dim3 grid((N + kCols - 1) / kCols, K / kBlock);
    hipLaunchKernelGGL(prepare_quant_asym_kernel, grid, dim3(kPrepThreads), 0, st, Wrot, lo, hi, K, N, norm,
                       static_cast<int8_t *>(codes), scales, zcw);
    return hipGetLastError();
}

// rowsum[i] = sum_k Xq[i][k]: one wave per token (the zero-point term of asymmetric weights needs it)
__global__ __launch_bounds__(256) void xq_rowsum_kernel(const int8_t *__restrict__ Xq, int64_t M, int K,
                                                        int32_t *__restrict__ rowsum)
{
    const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= M) return;
    const int lane = threadIdx.x & 63;
    const int8_t *row = Xq + i * K;
    int t = 0;
    for (int k = lane * 16; k < K; k += 64 * 16) {
        const int4 v = *reinterpret_cast<const int4 *>(row + k);
        const int wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int u = 0; u < 4; ++u)
            t += (int)(int8_t)(wv[u] & 0xFF) + (int)(int8_t)((wv[u] >> 8) & 0xFF) +
                 (int)(int8_t)((wv[u] >> 16) & 0xFF) + (wv[u] >> 24);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o);
    if (lane == 0) rowsum[i] = t;
}

hipError_t launch_xq_rowsum(const int8_t *Xq, int64_t M, int K, int32_t *rowsum, hipStream_t st)
{
    if (M <= 0) return hipSuccess;
    hipLaunchKernelGGL(xq_rowsum_kernel, dim3((unsigned)((M + 3) / 4)), dim3(256), 0, st, Xq, M, K, rowsum);
    return hipGetLastError();
}

hipError_t launch_weight_colsum(const void *codes, int K, int N, int32_t *colsum, hipStream_t st)
{
    hipLaunchKernelGGL(weight_colsum_kernel, dim3(N), dim3(64), 0, st, static_cast<const int8_t *>(codes), K, N, colsum);
    return hipGetLastError();
}

hipError_t launch_prepare_rotate(const float *W, int K, int N, const float *diag, const int32_t *perm,
                                 float *Wrot, float *amax, hipStream_t st)
{
    dim3 grid((N + kCols - 1) / kCols, K / kBlock);
    hipLaunchKernelGGL(prepare_rotate_kernel, grid, dim3(kPrepThreads), 0, st, W, K, N, diag, perm, Wrot, amax);
    return hipGetLastError();
}

// int4 weights: colsumw[n] = 16 * sum_g s_w[g][n] * (sum over the 128 codes of group g), one wave per
// output channel; a lane sums two packed bytes (four codes) per group.
__global__ __launch_bounds__(64) void weight_colsumw4_kernel(const uint8_t *__restrict__ codes, const float *__restrict__ scales,
                                                             int K, int N, float *__restrict__ colsumw)
{
    const int n = blockIdx.x, lane = threadIdx.x;
    const uint8_t *row = codes + (size_t)n * (K / 2);
    float t = 0.0f;
    for (int g = 0; g < K / kBlock; ++g) {
        // 64 bytes per group; lane takes byte `lane`: two codes as signed nibbles
        const uint32_t b = row[g * 64 + lane];
        int s = (int)((b & 0xF) ^ 8) - 8 + (int)(((b >> 4) & 0xF) ^ 8) - 8;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
        t += scales[(size_t)g * N + n] * (float)s;
    }
    if (lane == 0) colsumw[n] = 16.0f * t;
}

hipError_t launch_weight_colsumw4(const void *codes, const float *scales, int K, int N, float *colsumw, hipStream_t st)
{
    hipLaunchKernelGGL(weight_colsumw4_kernel, dim3(N), dim3(64), 0, st, static_cast<const uint8_t *>(codes), scales, K, N,
                       colsumw);
    return hipGetLastError();
}

hipError_t launch_prepare_rotate_dense(const float *W, int K, int N, const float *diag, const int32_t *perm,
                                       const float *R, float *Wrot, float *amax, hipStream_t st)
{
    dim3 grid((N + kCols - 1) / kCols, K / kBlock);
    hipLaunchKernelGGL(prepare_rotate_dense_kernel, grid, dim3(kPrepThreads), 0, st, W, K, N, diag, perm, R, Wrot, amax);
    return hipGetLastError();
}

hipError_t launch_prepare_quant(const float *Wrot, const float *amax, int K, int N, int wbits, float norm,
                                void *codes, float *scales, hipStream_t st)
{
    dim3 grid((N + kCols - 1) / kCols, K / kBlock);
    if (wbits == 8 || wbits == 6)
        hipLaunchKernelGGL(prepare_quant_kernel<8>, grid, dim3(kPrepThreads), 0, st, Wrot, amax, K, N, norm,
                           wbits == 8 ? 127.0f : 31.0f, codes, scales);
    else
        hipLaunchKernelGGL(prepare_quant_kernel<4>, grid, dim3(kPrepThreads), 0, st, Wrot, amax, K, N, norm, 7.0f, codes, scales);
    return hipGetLastError();
}

}  // namespace trdq
