// rotate_quant: G_t(X) = (X . Delta_t) . R of Eq. 10 followed by the per-token dynamic
// int8 quantiser (Eq. 1-2, symmetric form).  One streaming pass: 2 bytes in, 1 byte out
// per element, 4 bytes of scale per token.
//
// The pass is bound by the vector ALUs before it is bound by HBM (packed fp32 is not used),
// so the 128-point Walsh-Hadamard transform is split H_128 = H_16 (x) H_8 along the element
// index e = 8p + j and only the H_8 factor (three add stages over j, inside a lane) runs on
// the vector ALUs.  The H_16 factor over the chunk index p runs on the matrix cores as an
// exact fp32 product with a +-1 matrix (v_mfma_f32_16x16x4_f32, four chained instructions
// per j): products with +-1 are exact and the accumulation is fp32, so the result has the
// accuracy of fp32 butterflies.
//
// Mapping.  A workgroup owns 16 tokens; its NW waves split the K/128 blocks round-robin.
// For one block, lane (g = lane / 16, r = lane % 16) loads chunk p = 4s + g (16 bytes = 8
// channels) of token r in load s = 0..3, which is exactly the B-operand layout of the
// matrix instruction (k = g, n = r); the A operand is H_16[q][4s + g], a per-lane constant.
// The result leaves chunks q = 4g .. 4g+3 of token r in lane (g, r): 32 consecutive codes,
// two 16-byte stores.  A token's values stay in registers (at most SPW blocks per wave)
// until the token absmax is known: per-wave maxima are exchanged through LDS.
#include "device_utils.h"
#include "trdq_internal.h"

namespace trdq {

namespace {

constexpr int kTokensPerWG = 16;

template <int SPW, int MAXT>
__global__ __launch_bounds__(MAXT) void rotate_quant_kernel(
    const uint16_t *__restrict__ X, int64_t M, int nb, int64_t ldx,
    const float *__restrict__ diag, int8_t *__restrict__ Xq, float *__restrict__ sx,
    const uint4 *__restrict__ warm, int64_t warm_chunks)
{
    extern __shared__ __align__(16) float lds[];
    const int K = nb * kBlock;
    const int nw = blockDim.x >> 6;
    float *const d_s = lds;                          // [K] the group's diagonal
    float *const amax_s = lds + K;                   // [2][nw][16] per-wave token maxima (double-buffered)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, r = lane & 15;
    const int64_t groups = (M + kTokensPerWG - 1) / kTokensPerWG;

    // One raw block (64 bytes per lane) is always in flight: the wave walks the sequence
    // (group, block 0), (group, block 1), ..., (next group, block 0), ... and requests an item as
    // soon as the previous one has been unpacked.  Tokens past M are clamped to the last token:
    // they are rotated like the others (every lane takes part in the matrix instructions) and
    // never stored.
    uint4 raw[4];
    auto load_raw = [&](int i, int64_t tg) {
        // unconditional: a block index past the row or a group past the end is clamped to valid
        // memory (a redundant, cached read in the ragged / last step) and its data is not used
        int b = wave + nw * i;                       // wave-uniform
        if (b >= nb) b = nb - 1;
        int64_t token = tg * kTokensPerWG + r;
        if (token >= M) token = M - 1;
        const uint16_t *src = X + token * ldx + b * kBlock + g * 8;
#pragma unroll
        for (int s = 0; s < 4; ++s) raw[s] = *reinterpret_cast<const uint4 *>(src + s * 32);
    };

    int64_t tg = blockIdx.x;
    load_raw(0, tg);                                 // in flight while the diagonal is staged
    // Optional: read the next kernel's weights once (a couple of loads per lane, spread over the
    // whole grid).  Nothing waits for them before the end of the kernel; they only have to pass
    // through the memory-side cache so that the product kernel does not start on cold DRAM.
    uint32_t warm_acc = 0;
    for (int64_t c = (int64_t)blockIdx.x * blockDim.x + tid; c < warm_chunks; c += (int64_t)gridDim.x * blockDim.x) {
        const uint4 v = warm[c];
        warm_acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (diag) {
        for (int k = tid * 4; k < K; k += blockDim.x * 4)
            *reinterpret_cast<float4 *>(d_s + k) = *reinterpret_cast<const float4 *>(diag + k);
    } else {
        for (int k = tid * 4; k < K; k += blockDim.x * 4)
            *reinterpret_cast<float4 *>(d_s + k) = make_float4(1.f, 1.f, 1.f, 1.f);
    }
    __syncthreads();

    // A operand: H_16[q = r][p = 4s + g]
    float hs[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) hs[s] = (__builtin_popcount(r & (4 * s + g)) & 1) ? -1.0f : 1.0f;

    int parity = 0;
    for (; tg < groups; tg += gridDim.x) {
        const int64_t token = tg * kTokensPerWG + r;
        const bool token_ok = token < M;

        v4f out[SPW][8];   // out[i][j][q']: channel (4g + q') * 8 + j of block wave + nw*i, token r
        float amax = 0.0f;
#pragma unroll
        for (int i = 0; i < SPW; ++i) {
            const int b = wave + nw * i;
            if (b < nb) {
                float w[4][8];
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const float *dp = d_s + b * kBlock + (4 * s + g) * 8;
                    const float4 d0 = *reinterpret_cast<const float4 *>(dp);
                    const float4 d1 = *reinterpret_cast<const float4 *>(dp + 4);
                    const uint4 q = raw[s];
                    // scale by the diagonal fused into the first butterfly stage (pairs j, j+1)
                    const float t0 = bf16_hi(q.x) * d0.y, t1 = bf16_hi(q.y) * d0.w;
                    const float t2 = bf16_hi(q.z) * d1.y, t3 = bf16_hi(q.w) * d1.w;
                    float v[8];
                    v[0] = __builtin_fmaf(bf16_lo(q.x), d0.x, t0);
                    v[1] = __builtin_fmaf(bf16_lo(q.x), d0.x, -t0);
                    v[2] = __builtin_fmaf(bf16_lo(q.y), d0.z, t1);
                    v[3] = __builtin_fmaf(bf16_lo(q.y), d0.z, -t1);
                    v[4] = __builtin_fmaf(bf16_lo(q.z), d1.x, t2);
                    v[5] = __builtin_fmaf(bf16_lo(q.z), d1.x, -t2);
                    v[6] = __builtin_fmaf(bf16_lo(q.w), d1.z, t3);
                    v[7] = __builtin_fmaf(bf16_lo(q.w), d1.z, -t3);
                    // stages over index bits 1 and 2
                    const float a0 = v[0] + v[2], a2 = v[0] - v[2], a1 = v[1] + v[3], a3 = v[1] - v[3];
                    const float a4 = v[4] + v[6], a6 = v[4] - v[6], a5 = v[5] + v[7], a7 = v[5] - v[7];
                    w[s][0] = a0 + a4; w[s][4] = a0 - a4;
                    w[s][1] = a1 + a5; w[s][5] = a1 - a5;
                    w[s][2] = a2 + a6; w[s][6] = a2 - a6;
                    w[s][3] = a3 + a7; w[s][7] = a3 - a7;
                }
                // the raw buffer is free: request the next item of the sequence
                if (i + 1 < SPW) load_raw(i + 1, tg);
                else load_raw(0, tg + gridDim.x);
                // H_16 over the chunk index on the matrix cores: D[q][token] = sum_p H[q][p] * w[p][token]
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    v4f acc = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s = 0; s < 4; ++s)
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(hs[s], w[s][j], acc, 0, 0, 0);
                    out[i][j] = acc;
                    amax = fmaxf(fmaxf(amax, fabsf(acc[0])), fabsf(acc[1]));     // two v_max3_f32
                    amax = fmaxf(fmaxf(amax, fabsf(acc[2])), fabsf(acc[3]));
                }
            } else if (i + 1 == SPW) {
                load_raw(0, tg + gridDim.x);         // ragged last slot: still advance the sequence
            }
        }

        // token absmax: over the four lane-rows of this wave, then over the waves through LDS
        amax = fmaxf(amax, __shfl_xor(amax, 16));
        amax = fmaxf(amax, __shfl_xor(amax, 32));
        float *const am = amax_s + parity * nw * 16;
        if (g == 0) am[wave * 16 + r] = amax;
        __syncthreads();
        for (int wv = 0; wv < nw; ++wv) amax = fmaxf(amax, am[wv * 16 + r]);
        parity ^= 1;   // the next group writes the other buffer, so one barrier per group suffices

        // out holds sqrt(128) * V.  s_x = max|V| / 127; codes = rint(V / s_x) = rint(out * 127 / max|out|).
        const float inv = amax > 0.0f ? 127.0f / amax : 0.0f;
        if (wave == 0 && g == 0 && token_ok) sx[token] = amax * (0.08838834764831845f / 127.0f);

#pragma unroll
        for (int i = 0; i < SPW; ++i) {
            const int b = wave + nw * i;
            if (b < nb && token_ok) {
                uint32_t c[8];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    c[2 * q] = pack4_low_bytes(quant_bits(out[i][0][q], inv), quant_bits(out[i][1][q], inv),
                                               quant_bits(out[i][2][q], inv), quant_bits(out[i][3][q], inv));
                    c[2 * q + 1] = pack4_low_bytes(quant_bits(out[i][4][q], inv), quant_bits(out[i][5][q], inv),
                                                   quant_bits(out[i][6][q], inv), quant_bits(out[i][7][q], inv));
                }
                int8_t *dst = Xq + token * (int64_t)K + b * kBlock + g * 32;
                *reinterpret_cast<uint4 *>(dst) = make_uint4(c[0], c[1], c[2], c[3]);
                *reinterpret_cast<uint4 *>(dst + 16) = make_uint4(c[4], c[5], c[6], c[7]);
            }
        }
    }
    // keeps the loads above alive (never true: warm_chunks is not negative)
    if (warm_chunks < 0 && warm_acc == 0x9E3779B9u) sx[0] = 0.0f;
}

template <int SPW, int MAXT>
hipError_t launch_spw(const uint16_t *X, int64_t M, int nb, int nw, int64_t ldx, const float *diag,
                      int8_t *Xq, float *sx, const void *warm, int64_t warm_bytes, int wgs_per_cu, hipStream_t st)
{
    // persistent workgroups: a few per compute unit, each walking token groups
    const int64_t groups = (M + kTokensPerWG - 1) / kTokensPerWG;
    int64_t grid = (int64_t)256 * wgs_per_cu;
    if (grid > groups) grid = groups;
    const size_t smem = sizeof(float) * ((size_t)nb * kBlock + (size_t)2 * nw * 16);
    hipLaunchKernelGGL((rotate_quant_kernel<SPW, MAXT>), dim3((unsigned)grid), dim3(64 * nw), smem, st,
                       X, M, nb, ldx, diag, Xq, sx, static_cast<const uint4 *>(warm), warm ? warm_bytes / 16 : 0);
    return hipGetLastError();
}

}  // namespace

// Largest K: 12 waves x 3 blocks x 128 channels (a workgroup's waves must be co-resident, three
// per SIMD, which leaves 168 registers per lane: room for three blocks of results).
constexpr int kRQMaxBlocks = 36;

hipError_t launch_rotate_quant(const uint16_t *X, int64_t M, int K, int64_t ldx, const float *diag,
                               int8_t *Xq, float *sx, const void *warm, int64_t warm_bytes, hipStream_t st)
{
    if (M == 0) return hipSuccess;
    const int nb = K / kBlock;
    if (nb > kRQMaxBlocks) return launch_rotate_quant_wide(X, M, K, ldx, diag, Xq, sx, st);
    // three blocks per wave (two or one for narrow rows), then rebalance; workgroups of up to
    // 12 waves, as many per compute unit as 12 resident waves allow
    int spw = nb < 3 ? nb : 3;
    // few token groups (less than two workgroups per compute unit): spread each row over more
    // waves instead, so that the loads in flight still cover the memory latency
    const int64_t groups = (M + kTokensPerWG - 1) / kTokensPerWG;
    while (spw > 1 && groups * ((nb + spw - 1) / spw) < 256 * 8 && (nb + spw - 2) / (spw - 1) <= 12) --spw;
    const int nw = (nb + spw - 1) / spw;
    spw = (nb + nw - 1) / nw;
    const int wgs = 12 / nw > 0 ? 12 / nw : 1;
    const bool small = nw <= 4;      // up to 256 threads: no register cap from co-residency
    switch (spw) {
        case 1: return small ? launch_spw<1, 256>(X, M, nb, nw, ldx, diag, Xq, sx, warm, warm_bytes, wgs, st)
                             : launch_spw<1, 768>(X, M, nb, nw, ldx, diag, Xq, sx, warm, warm_bytes, wgs, st);
        case 2: return small ? launch_spw<2, 256>(X, M, nb, nw, ldx, diag, Xq, sx, warm, warm_bytes, wgs, st)
                             : launch_spw<2, 768>(X, M, nb, nw, ldx, diag, Xq, sx, warm, warm_bytes, wgs, st);
        default: return small ? launch_spw<3, 256>(X, M, nb, nw, ldx, diag, Xq, sx, warm, warm_bytes, wgs, st)
                              : launch_spw<3, 768>(X, M, nb, nw, ldx, diag, Xq, sx, warm, warm_bytes, wgs, st);
    }
}

}  // namespace trdq
