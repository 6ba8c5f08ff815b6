// rotate_quant for wide inputs (K > 4608): the all-vector-ALU form of the rotate + quantise
// pass (see rotate_quant.hip for the operation).
//
// Mapping.  A 128-channel rotation block is held by a row of 16 lanes (8 consecutive
// channels per lane = one 16-byte load).  A wave of 64 lanes is four such rows.  S of the
// four lane-rows share one token and take its blocks round-robin (block = t*S + s), each
// lane-row handling T blocks, so a token's K = 128*S*T channels stay in registers between
// the rotation and the quantisation: X is read exactly once and nothing goes through LDS.
// The butterflies of index bits 0-2 run inside a lane, bits 3-6 across lanes with DPP moves.
// The token absmax is a DPP max over 16 lanes plus (S > 1) a cross-row exchange.
#include "rotate_core.h"

namespace trdq {

namespace {

constexpr int kRQThreads = 256;

template <int T, int S>
__global__ __launch_bounds__(kRQThreads) void rotate_quant_kernel(
    const uint16_t *__restrict__ X, int64_t M, int nb, int64_t ldx,
    const float *__restrict__ diag, int8_t *__restrict__ Xq, float *__restrict__ sx)
{
    constexpr int kTokensPerWave = 4 / S;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int p = lane & 15;       // position inside the block: channels 8p .. 8p+7
    const int lrow = lane >> 4;    // lane-row 0..3
    const int s = lrow % S;        // which share of the token's blocks
    const int64_t token = ((int64_t)blockIdx.x * (kRQThreads / 64) + wave) * kTokensPerWave + lrow / S;
    const bool token_ok = token < M;
    const int K = nb * kBlock;
    const LaneSigns sg(p);

    float v[T][8];
    float amax;
    rotate_token<T, S>(X + token * ldx, token_ok, nb, s, p, diag, sg, v, amax);
    const float inv = token_inv_scale(amax);
    if (token_ok && s == 0 && p == 0) sx[token] = token_scale(amax);

#pragma unroll
    for (int t = 0; t < T; ++t) {
        const int b = t * S + s;
        if (token_ok && b < nb)
            *reinterpret_cast<uint2 *>(Xq + token * (int64_t)K + (int64_t)b * kBlock + p * 8) =
                quant_pack8(v[t], inv);
    }
}

template <int T, int S>
hipError_t launch_ts(const uint16_t *X, int64_t M, int nb, int64_t ldx, const float *diag,
                     int8_t *Xq, float *sx, hipStream_t st)
{
    const int64_t tokens_per_wg = (kRQThreads / 64) * (4 / S);
    const int64_t grid = (M + tokens_per_wg - 1) / tokens_per_wg;
    hipLaunchKernelGGL((rotate_quant_kernel<T, S>), dim3((unsigned)grid), dim3(kRQThreads), 0, st,
                       X, M, nb, ldx, diag, Xq, sx);
    return hipGetLastError();
}

template <int S>
hipError_t launch_s(int T, const uint16_t *X, int64_t M, int nb, int64_t ldx, const float *diag,
                    int8_t *Xq, float *sx, hipStream_t st)
{
    switch (T) {
#define TRDQ_RQ_CASE(TT) case TT: return launch_ts<TT, S>(X, M, nb, ldx, diag, Xq, sx, st);
        TRDQ_RQ_CASE(1) TRDQ_RQ_CASE(2) TRDQ_RQ_CASE(3) TRDQ_RQ_CASE(4) TRDQ_RQ_CASE(5)
        TRDQ_RQ_CASE(6) TRDQ_RQ_CASE(7) TRDQ_RQ_CASE(8) TRDQ_RQ_CASE(9) TRDQ_RQ_CASE(10)
        TRDQ_RQ_CASE(11) TRDQ_RQ_CASE(12) TRDQ_RQ_CASE(13) TRDQ_RQ_CASE(14) TRDQ_RQ_CASE(15)
        TRDQ_RQ_CASE(16)
#undef TRDQ_RQ_CASE
    }
    return hipErrorInvalidValue;
}

}  // namespace

// Largest K the register-resident kernel takes: 4 lane-rows x 16 blocks x 128 channels.
constexpr int kRQMaxBlocks = 64;

hipError_t launch_rotate_quant_wide(const uint16_t *X, int64_t M, int K, int64_t ldx, const float *diag,
                               int8_t *Xq, float *sx, hipStream_t st)
{
    if (M == 0) return hipSuccess;
    const int nb = K / kBlock;
    if (nb > kRQMaxBlocks) return hipErrorInvalidValue;
    // S lane-rows per token: as few as keep T = ceil(nb / S) <= 12 registers-blocks per lane
    int S = 1;
    while (S < 4 && (nb + S - 1) / S > 12) S *= 2;
    const int T = (nb + S - 1) / S;
    if (S == 1) return launch_s<1>(T, X, M, nb, ldx, diag, Xq, sx, st);
    if (S == 2) return launch_s<2>(T, X, M, nb, ldx, diag, Xq, sx, st);
    return launch_s<4>(T, X, M, nb, ldx, diag, Xq, sx, st);
}

}  // namespace trdq
