// rotate_quant_rpr: the full activation transform of Eq. 9,
//   G_t(X) = (X . Delta_t) . R^(1) . P . R^(2),
// first block rotation, zigzag permutation P (Sec. 3.2), second block rotation, followed by the
// per-token dynamic int8 quantiser (Eq. 1-2, symmetric form).  Both rotations use the same
// block-diagonal Hadamard blocks as rotate_quant; (U P)[k'] = U[perm[k']].
//
// The permutation moves channels between blocks, so a token's whole rotated row has to exist
// before the second rotation starts: a workgroup owns TOK tokens and keeps their first-rotation
// output in LDS as fp32 (TOK x K x 4 bytes: 16 tokens up to K = 2304, 8 tokens up to K = 4608).
//   stage 1: each wave rotates its blocks of the row (H_128 = H_16 (x) H_8: the H_8 factor and the
//            diagonal on the vector ALU inside a lane, the H_16 factor over the 16 chunks of a
//            block as an exact fp32 product with a +-1 matrix, v_mfma_f32_16x16x4_f32) and
//            writes the result to LDS by channel;
//   stage 2: each wave gathers the channels perm[k'] of its output blocks from LDS, rotates them
//            the same way and keeps the results in registers until the token maxima are known
//            (exchanged through LDS), then quantises and stores like rotate_quant.
// The matrix instruction has 16 columns: 16 tokens of one block, or, with TOK = 8, 8 tokens of
// two blocks at once (lanes r >= 8 hold token r - 8 of the wave's second block; the +-1 operand
// is the same for every column).  Both rotations are unnormalised; the factor 1/128 goes into
// the scale.  Entries of perm are clamped to [0, K) on the way in, so a bad table gives wrong
// numbers, never an access outside the row.
#include "device_utils.h"
#include "trdq_internal.h"

namespace trdq {

namespace {

constexpr int kRowPad = 4;     // floats of padding per LDS row: tokens land in different banks

// in-lane H_8 over 8 values (three add stages)
__device__ __forceinline__ void h8(float (&v)[8])
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

template <int TOK, int SPW>
__global__ __launch_bounds__(768) void rotate_quant_rpr_kernel(
    const uint16_t *__restrict__ X, int64_t M, int nb, int64_t ldx,
    const float *__restrict__ diag, const int32_t *__restrict__ perm,
    int8_t *__restrict__ Xq, float *__restrict__ sx, int32_t *__restrict__ zc,
    const uint4 *__restrict__ warm, int64_t warm_chunks)
{
    // zc != null: the asymmetric quantiser of Eq. 1-3 (codes stored as q - 128, zc[i] = 128 - z_i), as in rotate_quant
    static_assert(TOK == 16 || TOK == 8, "16 or 8 tokens per workgroup");
    const bool asym = zc != nullptr;
    extern __shared__ __align__(16) float lds[];
    const int K = nb * kBlock;
    const int nw = blockDim.x >> 6;
    const int rowf = K + kRowPad;                    // floats per LDS row
    float *const T = lds;                            // [TOK][rowf]: first-rotation output
    float *const amax_s = lds + (size_t)TOK * rowf;  // [2][nw][16] (maxima, minima); after it a 1 KB dump area for the weight copies

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, r = lane & 15;
    constexpr int BPI = 16 / TOK;                    // blocks a wave rotates per matrix instruction
    const int rt = r & (TOK - 1);                    // token slot of this lane
    const int bsel = r / TOK;                        // which of the item's blocks this lane holds
    const int64_t tg = blockIdx.x;
    int64_t token = tg * TOK + rt;
    const bool token_ok = token < M;
    if (token >= M) token = M - 1;                   // clamped: rotated like the others, never stored

    // ---- stage 1: T[token][.] = (x * d) H_128 per block (natural row order of H_16) -----------
    float hn[4];                                     // A operand: H_16[q = r][p = 4s + g]
#pragma unroll
    for (int s = 0; s < 4; ++s) hn[s] = (__builtin_popcount(r & (4 * s + g)) & 1) ? -1.0f : 1.0f;
#pragma unroll
    for (int i = 0; i < SPW; ++i) {
        const int b0 = (wave + nw * i) * BPI;        // wave-uniform: first block of the item
        if (b0 < nb) {
            const int bl = b0 + bsel;                // this lane's block (may be one past the end)
            const bool b_ok = bl < nb;
            const int b = b_ok ? bl : nb - 1;        // clamped: rotated, not written
            float w[4][8];
            const uint16_t *src = X + token * ldx + b * kBlock + g * 8;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const uint4 q = *reinterpret_cast<const uint4 *>(src + s * 32);
                float4 d0 = make_float4(1.f, 1.f, 1.f, 1.f), d1 = d0;
                if (diag) {
                    const float *dp = diag + b * kBlock + (4 * s + g) * 8;
                    d0 = *reinterpret_cast<const float4 *>(dp);
                    d1 = *reinterpret_cast<const float4 *>(dp + 4);
                }
                w[s][0] = bf16_lo(q.x) * d0.x; w[s][1] = bf16_hi(q.x) * d0.y;
                w[s][2] = bf16_lo(q.y) * d0.z; w[s][3] = bf16_hi(q.y) * d0.w;
                w[s][4] = bf16_lo(q.z) * d1.x; w[s][5] = bf16_hi(q.z) * d1.y;
                w[s][6] = bf16_lo(q.w) * d1.z; w[s][7] = bf16_hi(q.w) * d1.w;
                h8(w[s]);
            }
            // D[q][token] = sum_p H_16[q][p] * w[p][token]; lane (g, r) receives q = 4g .. 4g+3
            v4f acc[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                acc[j] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(hn[s], w[s][j], acc[j], 0, 0, 0);
            }
            if (b_ok) {
                float *dst = T + (size_t)rt * rowf + b * kBlock + g * 32;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    *reinterpret_cast<float4 *>(dst + q * 8) = make_float4(acc[0][q], acc[1][q], acc[2][q], acc[3][q]);
                    *reinterpret_cast<float4 *>(dst + q * 8 + 4) = make_float4(acc[4][q], acc[5][q], acc[6][q], acc[7][q]);
                }
            }
        }
    }
    // Optional: pull the following product's weight codes through the memory-side cache (see
    // rotate_quant): up to four direct-to-LDS copies per wave into a dump area nobody reads.
    if (warm_chunks > 0) {
        const uint32_t dump = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) float *)lds +
                              (uint32_t)(sizeof(float) * ((size_t)TOK * rowf + (size_t)nw * 32));
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int64_t c0 = ((int64_t)t * gridDim.x + blockIdx.x) * blockDim.x + (wave << 6);   // wave-uniform
            if (c0 < warm_chunks) {
                int64_t c = c0 + lane;
                if (c >= warm_chunks) c = warm_chunks - 1;
                asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                             :: "v"((uint32_t)(c << 4)), "s"(warm), "s"(dump) : "memory", "m0");
            }
        }
    }
    __syncthreads();

    // ---- stage 2: gather by perm, rotate again, keep in registers -----------------------------------
    // Rows of H_16 permuted as in rotate_quant: lane group g' receives chunks 2g', 2g'+1 (i = 0, 1)
    // and 8 + 2g', 9 + 2g' (i = 2, 3), so each 16-byte store covers 64 consecutive bytes of a token.
    const int qrow = (r & 2) ? 8 + 2 * (r >> 2) + (r & 1) : 2 * (r >> 2) + (r & 1);
    float hs[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) hs[s] = (__builtin_popcount(qrow & (4 * s + g)) & 1) ? -1.0f : 1.0f;

    v4f out[SPW][8];
    float amax = 0.0f;
    float amin = 0.0f;                               // asymmetric: the token minimum (<= 0); amax is then the maximum (>= 0)
    const float *Trow = T + (size_t)rt * rowf;
#pragma unroll
    for (int i = 0; i < SPW; ++i) {
        const int b0 = (wave + nw * i) * BPI;
        if (b0 < nb) {
            const int b = (b0 + bsel < nb) ? b0 + bsel : nb - 1;
            float w[4][8];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int32_t *pp = perm + b * kBlock + (4 * s + g) * 8;
                const int4 i0 = *reinterpret_cast<const int4 *>(pp);
                const int4 i1 = *reinterpret_cast<const int4 *>(pp + 4);
                const int idx[8] = {i0.x, i0.y, i0.z, i0.w, i1.x, i1.y, i1.z, i1.w};
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    int k = idx[j];
                    k = k < 0 ? 0 : (k >= K ? K - 1 : k);
                    w[s][j] = Trow[k];
                }
                h8(w[s]);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                v4f acc = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(hs[s], w[s][j], acc, 0, 0, 0);
                out[i][j] = acc;
                if (asym) {
                    amax = fmaxf(fmaxf(amax, fmaxf(acc[0], acc[1])), fmaxf(acc[2], acc[3]));
                    amin = fminf(fminf(amin, fminf(acc[0], acc[1])), fminf(acc[2], acc[3]));
                } else {
                    amax = fmaxf(fmaxf(amax, fabsf(acc[0])), fabsf(acc[1]));
                    amax = fmaxf(fmaxf(amax, fabsf(acc[2])), fabsf(acc[3]));
                }
            }
        }
    }

    // token absmax: over the four lane-rows of this wave, then over the waves through LDS
    amax = fmaxf(amax, __shfl_xor(amax, 16));
    amax = fmaxf(amax, __shfl_xor(amax, 32));
    if (BPI == 2) amax = fmaxf(amax, __shfl_xor(amax, 8));       // the token's other block in this wave
    amin = fminf(amin, __shfl_xor(amin, 16));
    amin = fminf(amin, __shfl_xor(amin, 32));
    if (BPI == 2) amin = fminf(amin, __shfl_xor(amin, 8));
    if (g == 0) {
        amax_s[wave * 16 + r] = amax;
        amax_s[(nw + wave) * 16 + r] = amin;
    }
    __syncthreads();
    for (int wv = 0; wv < nw; ++wv) {
        amax = fmaxf(amax, amax_s[wv * 16 + r]);
        amin = fminf(amin, amax_s[(nw + wv) * 16 + r]);
    }

    // out holds 128 * V.  Symmetric: s_x = max|V| / 127; codes = rint(V / s_x) = rint(out * 127 / max|out|).
    // Asymmetric (range [lo, hi] with lo <= 0 <= hi): s_x = (hi - lo) / 255, z = -rint(lo / s_x), stored code =
    // clamp(rint(V / s_x) + z, 0, 255) - 128; the integer offset rides in the rounding constant of the same FMA.
    float inv, magic = kRoundMagic;
    if (asym) {
        const float range = amax - amin;
        inv = range > 0.0f ? 255.0f / range : 0.0f;
        const float z = -rintf(amin * inv);
        magic = kRoundMagic + (z - 128.0f);
        if (wave == 0 && g == 0 && r < TOK && token_ok) {
            sx[token] = range * (0.0078125f / 255.0f);
            zc[token] = 128 - (int)z;
        }
    } else {
        inv = amax > 0.0f ? 127.0f / amax : 0.0f;
        if (wave == 0 && g == 0 && r < TOK && token_ok) sx[token] = amax * (0.0078125f / 127.0f);
    }
    auto code_bits = [&](float v) -> uint32_t {
        const float t = __builtin_fmaf(v, inv, magic);
        // symmetric codes cannot leave +-127; the clamp only acts on the asymmetric range ends
        return __float_as_uint(__builtin_amdgcn_fmed3f(t, kRoundMagic - 128.0f, kRoundMagic + 127.0f));
    };

#pragma unroll
    for (int i = 0; i < SPW; ++i) {
        const int b = (wave + nw * i) * BPI + bsel;
        if (b < nb && token_ok) {
            uint32_t c[8];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                c[2 * q] = pack4_low_bytes(code_bits(out[i][0][q]), code_bits(out[i][1][q]),
                                           code_bits(out[i][2][q]), code_bits(out[i][3][q]));
                c[2 * q + 1] = pack4_low_bytes(code_bits(out[i][4][q]), code_bits(out[i][5][q]),
                                               code_bits(out[i][6][q]), code_bits(out[i][7][q]));
            }
            int8_t *dst = Xq + token * (int64_t)K + b * kBlock + g * 16;
            *reinterpret_cast<uint4 *>(dst) = make_uint4(c[0], c[1], c[2], c[3]);
            *reinterpret_cast<uint4 *>(dst + 64) = make_uint4(c[4], c[5], c[6], c[7]);
        }
    }
    // the copies to the dump area must have landed before the workgroup's LDS is given away
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

template <int TOK, int SPW>
hipError_t launch_rpr(const uint16_t *X, int64_t M, int nb, int nw, int64_t ldx, const float *diag,
                      const int32_t *perm, int8_t *Xq, float *sx, int32_t *zc, const void *warm, int64_t warm_bytes,
                      hipStream_t st)
{
    const int K = nb * kBlock;
    const size_t smem = sizeof(float) * ((size_t)TOK * (K + kRowPad) + (size_t)nw * 32) + 1024;
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(rotate_quant_rpr_kernel<TOK, SPW>), 160 * 1024);
        e != hipSuccess)
        return e;
    const int64_t groups = (M + TOK - 1) / TOK;
    hipLaunchKernelGGL((rotate_quant_rpr_kernel<TOK, SPW>), dim3((unsigned)groups), dim3(64 * nw), smem, st,
                       X, M, nb, ldx, diag, perm, Xq, sx, zc, static_cast<const uint4 *>(warm),
                       (warm && warm_bytes < ((int64_t)1 << 32)) ? warm_bytes / 16 : 0);
    return hipGetLastError();
}

}  // namespace

// K up to 4608 (36 blocks): 12 waves x 3 blocks; LDS holds 8 tokens x 4608 floats.
bool rotate_quant_rpr_supports(int K) { return K > 0 && K % kBlock == 0 && K / kBlock <= 36; }

hipError_t launch_rotate_quant_rpr(const uint16_t *X, int64_t M, int K, int64_t ldx, const float *diag,
                                   const int32_t *perm, int8_t *Xq, float *sx, const void *warm, int64_t warm_bytes,
                                   hipStream_t st, int32_t *zc)
{
    if (M == 0) return hipSuccess;
    if (!rotate_quant_rpr_supports(K)) return hipErrorInvalidValue;
    const int nb = K / kBlock;
    // 16 tokens per workgroup while their rows fit LDS, else 8 tokens and two blocks per item
    const bool tok16 = (size_t)16 * (K + kRowPad) * 4 + (size_t)12 * 128 + 1024 <= 150 * 1024;
    const int items = tok16 ? nb : (nb + 1) / 2;
    const int spw = items <= 12 ? 1 : (items <= 24 ? 2 : 3);
    const int nw = (items + spw - 1) / spw;
    if (tok16) {
        switch (spw) {
            case 1: return launch_rpr<16, 1>(X, M, nb, nw, ldx, diag, perm, Xq, sx, zc, warm, warm_bytes, st);
            case 2: return launch_rpr<16, 2>(X, M, nb, nw, ldx, diag, perm, Xq, sx, zc, warm, warm_bytes, st);
            default: return launch_rpr<16, 3>(X, M, nb, nw, ldx, diag, perm, Xq, sx, zc, warm, warm_bytes, st);
        }
    }
    switch (spw) {
        case 1: return launch_rpr<8, 1>(X, M, nb, nw, ldx, diag, perm, Xq, sx, zc, warm, warm_bytes, st);
        case 2: return launch_rpr<8, 2>(X, M, nb, nw, ldx, diag, perm, Xq, sx, zc, warm, warm_bytes, st);
        default: return launch_rpr<8, 3>(X, M, nb, nw, ldx, diag, perm, Xq, sx, zc, warm, warm_bytes, st);
    }
}

}  // namespace trdq
