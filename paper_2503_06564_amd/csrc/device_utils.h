// Device helpers for the gfx950 kernels: lane exchange inside a row of 16 lanes,
// the block-128 Walsh-Hadamard butterflies, int8 packing and bf16 conversion.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace trdq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

// ---- data-parallel-primitive moves inside a row of 16 lanes -------------------------
// DPP control words: quad_perm = p0 | p1<<2 | p2<<4 | p3<<6, row_ror:n = 0x120 + n,
// row_mirror = 0x140, row_half_mirror = 0x141.
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppQuadRev = 0x1B;     // quad_perm [3,2,1,0]   : lane ^ 3
constexpr int kDppHalfMirror = 0x141; // lane -> 7 - lane in 8  : lane ^ 7
constexpr int kDppRor8 = 0x128;       // (lane + 8) % 16        : lane ^ 8

template <int CTRL>
__device__ __forceinline__ float dpp_f(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}

// value of lane (l ^ MASK), MASK in {1, 2, 4, 8}, l = lane index inside its row of 16
template <int MASK>
__device__ __forceinline__ float row_xor(float x)
{
    if constexpr (MASK == 1) return dpp_f<kDppXor1>(x);
    else if constexpr (MASK == 2) return dpp_f<kDppXor2>(x);
    else if constexpr (MASK == 4) return dpp_f<kDppHalfMirror>(dpp_f<kDppQuadRev>(x));  // ^3 then ^7
    else return dpp_f<kDppRor8>(x);
}

// ---- Walsh-Hadamard transform of one 128-element block --------------------------------
// Natural (Sylvester) order, unnormalised: out[j] = sum_k in[k] * (-1)^popcount(j & k).
// The block lives in 16 lanes, lane p (0..15) holding elements 8p .. 8p+7.
// Index bits 0-2 are handled inside the lane, bits 3-6 across lanes p ^ {1,2,4,8}.
__device__ __forceinline__ void fwht8_inlane(float (&v)[8])
{
#pragma unroll
    for (int h = 1; h < 8; h <<= 1) {
#pragma unroll
        for (int i = 0; i < 8; i += 2 * h) {
#pragma unroll
            for (int j = i; j < i + h; ++j) {
                float a = v[j], b = v[j + h];
                v[j] = a + b;
                v[j + h] = a - b;
            }
        }
    }
}

// sign[m] = 0x80000000 when bit m of the lane's position p is set (the lane holds the
// "b" side of the butterfly and must produce a - b = partner - own).
struct LaneSigns {
    uint32_t s1, s2, s4, s8;
    __device__ __forceinline__ explicit LaneSigns(int p)
        : s1((uint32_t)(p & 1) << 31), s2((uint32_t)(p & 2) << 30),
          s4((uint32_t)(p & 4) << 29), s8((uint32_t)(p & 8) << 28) {}
};

template <int MASK>
__device__ __forceinline__ float butterfly_xlane(float own, uint32_t sign)
{
    float partner = row_xor<MASK>(own);
    return partner + __uint_as_float(__float_as_uint(own) ^ sign);
}

__device__ __forceinline__ void fwht128_rows16(float (&v)[8], const LaneSigns &sg)
{
    fwht8_inlane(v);
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = butterfly_xlane<1>(v[j], sg.s1);
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = butterfly_xlane<2>(v[j], sg.s2);
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = butterfly_xlane<4>(v[j], sg.s4);
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = butterfly_xlane<8>(v[j], sg.s8);
}

// max over the 16 lanes of a row (every lane gets the result)
__device__ __forceinline__ float row16_max(float x)
{
    x = fmaxf(x, row_xor<1>(x));
    x = fmaxf(x, row_xor<2>(x));
    x = fmaxf(x, row_xor<4>(x));
    x = fmaxf(x, row_xor<8>(x));
    return x;
}

// ---- rounding to int8 and packing -------------------------------------------------------
// fma(v, inv, 1.5 * 2^23) rounds v * inv to the nearest integer (ties to even, one rounding)
// and leaves its two's-complement low byte in the low byte of the float's bit pattern
// (valid for |v * inv| < 2^22).
constexpr float kRoundMagic = 12582912.0f;

__device__ __forceinline__ uint32_t quant_bits(float v, float inv)
{
    return __float_as_uint(__builtin_fmaf(v, inv, kRoundMagic));
}

// low bytes of four words -> one dword (a in bits 0-7 ... d in bits 24-31)
__device__ __forceinline__ uint32_t pack4_low_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    uint32_t ab = __builtin_amdgcn_perm(b, a, 0x0c0c0400u);  // [a.b0, b.b0, 0, 0]
    uint32_t cd = __builtin_amdgcn_perm(d, c, 0x0c0c0400u);  // [c.b0, d.b0, 0, 0]
    return __builtin_amdgcn_perm(cd, ab, 0x05040100u);       // [ab.b0, ab.b1, cd.b0, cd.b1]
}

// ---- bf16 ---------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// float32 -> bf16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// two float32 -> packed bf16 pair (lo in bits 0-15), round to nearest even: one
// v_cvt_pk_bf16_f32 on gfx950
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// 16-byte store of finished output
__device__ __forceinline__ void store_out16(void *p, uint4 v) { *reinterpret_cast<uint4 *>(p) = v; }

}  // namespace trdq
