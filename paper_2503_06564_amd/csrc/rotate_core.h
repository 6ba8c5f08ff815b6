// Per-token rotation core shared by the streaming rotate_quant kernel and the fused
// linear kernel: a row of 16 lanes rotates T blocks of one token and keeps them in registers.
#pragma once

#include "device_utils.h"
#include "trdq_internal.h"

namespace trdq {

// Loads block b = t*S + s (t < T) of one token (8 channels per lane), applies the diagonal,
// runs the block-128 Walsh-Hadamard butterflies and tracks max |v|.  v = sqrt(128) * V.
// Lanes whose token or block is out of range carry zeros (and still take part in the lane
// exchanges, which need the whole wave).
// RANGE: track the signed extremes instead (amax = max(0, max v), amin = min(0, min v)), which is
// what the asymmetric quantiser of Eq. 1-3 needs.
template <int T, int S, bool RANGE = false>
__device__ __forceinline__ void rotate_token(const uint16_t *__restrict__ xtok, bool token_ok, int nb,
                                             int s, int p, const float *__restrict__ diag,
                                             const LaneSigns &sg, float (&v)[T][8], float &amax, float &amin)
{
    amax = 0.0f;
    amin = 0.0f;
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const int b = t * S + s;
        const bool ok = token_ok && b < nb;
        uint4 raw = make_uint4(0, 0, 0, 0);
        float4 d0 = make_float4(1.f, 1.f, 1.f, 1.f), d1 = d0;
        if (ok) {
            raw = *reinterpret_cast<const uint4 *>(xtok + (int64_t)b * kBlock + p * 8);
            if (diag) {
                d0 = *reinterpret_cast<const float4 *>(diag + b * kBlock + p * 8);
                d1 = *reinterpret_cast<const float4 *>(diag + b * kBlock + p * 8 + 4);
            }
        }
        v[t][0] = bf16_lo(raw.x) * d0.x;
        v[t][1] = bf16_hi(raw.x) * d0.y;
        v[t][2] = bf16_lo(raw.y) * d0.z;
        v[t][3] = bf16_hi(raw.y) * d0.w;
        v[t][4] = bf16_lo(raw.z) * d1.x;
        v[t][5] = bf16_hi(raw.z) * d1.y;
        v[t][6] = bf16_lo(raw.w) * d1.z;
        v[t][7] = bf16_hi(raw.w) * d1.w;
        fwht128_rows16(v[t], sg);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if constexpr (RANGE) {
                amax = fmaxf(amax, v[t][j]);
                amin = fminf(amin, v[t][j]);
            } else {
                amax = fmaxf(amax, fabsf(v[t][j]));
            }
        }
    }
    amax = row16_max(amax);
    if constexpr (S >= 2) amax = fmaxf(amax, __shfl_xor(amax, 16));
    if constexpr (S >= 4) amax = fmaxf(amax, __shfl_xor(amax, 32));
    if constexpr (RANGE) {
        amin = -row16_max(-amin);
        if constexpr (S >= 2) amin = fminf(amin, __shfl_xor(amin, 16));
        if constexpr (S >= 4) amin = fminf(amin, __shfl_xor(amin, 32));
    }
}

template <int T, int S>
__device__ __forceinline__ void rotate_token(const uint16_t *__restrict__ xtok, bool token_ok, int nb,
                                             int s, int p, const float *__restrict__ diag,
                                             const LaneSigns &sg, float (&v)[T][8], float &amax)
{
    float unused;
    rotate_token<T, S, false>(xtok, token_ok, nb, s, p, diag, sg, v, amax, unused);
}

// v holds sqrt(128) * V.  s_x = max|V| / 127; codes = rint(V / s_x) = rint(v * 127 / max|v|).
__device__ __forceinline__ float token_inv_scale(float amax) { return amax > 0.0f ? 127.0f / amax : 0.0f; }
__device__ __forceinline__ float token_scale(float amax) { return amax * (0.08838834764831845f / 127.0f); }

// eight codes of one lane as 8 bytes, channel order
__device__ __forceinline__ uint2 quant_pack8(const float (&v)[8], float inv)
{
    uint2 out;
    out.x = pack4_low_bytes(quant_bits(v[0], inv), quant_bits(v[1], inv),
                            quant_bits(v[2], inv), quant_bits(v[3], inv));
    out.y = pack4_low_bytes(quant_bits(v[4], inv), quant_bits(v[5], inv),
                            quant_bits(v[6], inv), quant_bits(v[7], inv));
    return out;
}

// Asymmetric per-token quantiser (Eq. 1-3) of a token whose rotated values span [lo, hi] with
// lo <= 0 <= hi (v = sqrt(128) * V): s_x = (hi - lo) / 255, z = -rint(lo / s_x), stored code =
// clamp(rint(V / s_x) + z, 0, 255) - 128.  The integer offset z - 128 rides in the rounding
// constant of the FMA that scales the value.
struct TokenRangeQuant {
    float inv, magic, scale;
    int zc;                     // 128 - z: what multiplies the weights' column sums in the epilogue
    __device__ __forceinline__ TokenRangeQuant(float lo, float hi)
    {
        const float range = hi - lo;
        inv = range > 0.0f ? 255.0f / range : 0.0f;
        const float z = -rintf(lo * inv);
        magic = kRoundMagic + (z - 128.0f);
        scale = range * (0.08838834764831845f / 255.0f);
        zc = 128 - (int)z;
    }
    __device__ __forceinline__ uint32_t bits(float v) const
    {
        const float t = __builtin_fmaf(v, inv, magic);
        return __float_as_uint(__builtin_amdgcn_fmed3f(t, kRoundMagic - 128.0f, kRoundMagic + 127.0f));
    }
    __device__ __forceinline__ uint2 pack8(const float (&v)[8]) const
    {
        uint2 out;
        out.x = pack4_low_bytes(bits(v[0]), bits(v[1]), bits(v[2]), bits(v[3]));
        out.y = pack4_low_bytes(bits(v[4]), bits(v[5]), bits(v[6]), bits(v[7]));
        return out;
    }
};

}  // namespace trdq
