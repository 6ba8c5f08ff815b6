// rotate_quant: G_t(X) = (X . Delta_t) . R of Eq. 10 followed by the per-token dynamic
// int8 quantiser (Eq. 1-2, symmetric form).  One streaming pass: 2 bytes in, 1 byte out
// per element, 4 bytes of scale per token.
//
// The pass is bound by the vector ALUs before it is bound by HBM (packed fp32 is not used, and
// an fp32 matrix instruction keeps the vector ALU of its SIMD busy: nothing else issues under
// it), so as much of the transform as can be made exact runs on the bf16 matrix pipe, which does
// overlap with vector work.  The 128-point Walsh-Hadamard transform is split
// H_128 = H_16 (x) H_8 along the element index e = 8p + j:
//
//   u[q][j] = sum_p H_16[q][p] * d[8p + j] * x[8p + j]      (matrix pipe, K = 16 = all p)
//   y[8q + j'] = sum_j H_8[j'][j] * u[q][j]                 (three add stages inside a lane)
//
// x is bf16 as it comes from memory: it is the B operand without any conversion.  The A operand
// is H_16[q][p] * d[8p + j]: the fp32 diagonal is cut into three bf16 pieces d = d_hi + d_mid +
// d_lo (8 + 8 + 8 mantissa bits, exact), one v_mfma_f32_16x16x16_bf16 per piece accumulating
// into the same fp32 registers.  Every product is exact (8 x 8 bits) and the accumulation is
// fp32, so the result has the accuracy of fp32 butterflies applied to d * x.
//
// Mapping.  A workgroup owns 16 tokens; its NW waves split the K/128 blocks round-robin.
// For one block, lane (g = lane / 16, r = lane % 16) loads chunk p = 4s + g (16 bytes = 8
// channels j) of token r in load s = 0..3.  Element j of the four loads, picked out with two
// byte permutes, is the B operand (k = 4g + s <-> p = 4s + g, n = r) of the instruction for j.
// The pieces of d, in the same k order, are staged once per workgroup in LDS; a lane reads the
// four of its group g with one 8-byte read and applies the signs of its row of H_16 with two
// XORs.  The rows of H_16 are permuted so that the result leaves chunks 2g, 2g+1 and 8+2g, 9+2g
// of token r in lane (g, r): two 16-byte stores, each of which covers 64 consecutive bytes of
// the token over the four lanes that share r.  A token's values stay in registers (at most SPW
// blocks per wave) until the token absmax is known: per-wave maxima are exchanged through LDS.
#include <type_traits>

#include "device_utils.h"
#include "trdq_internal.h"

namespace trdq {

namespace {

constexpr int kTokensPerWG = 16;

typedef short v4s __attribute__((ext_vector_type(4)));

// LDS bytes of the diagonal's pieces: [block][j][piece][g] x 4 bf16 (k = 4g .. 4g+3)
__host__ __device__ constexpr size_t diag_table_bytes(int nb) { return (size_t)nb * 8 * 3 * 4 * 8; }

// ASYM: the asymmetric quantiser of Eq. 1-3 instead (per-token minimum and maximum, zero point):
// codes q in 0..255 are stored as q - 128 so that they stay int8 for the matrix instruction, and
// zc[i] = 128 - z_i is what the product's epilogue needs with the weights' column sums.
template <int SPW, int MAXT, bool ASYM>
__global__ __launch_bounds__(MAXT) void rotate_quant_kernel(
    const uint16_t *__restrict__ X, int64_t M, int nb, int64_t ldx,
    const float *__restrict__ diag, int8_t *__restrict__ Xq, float *__restrict__ sx,
    int32_t *__restrict__ zc, const uint4 *__restrict__ warm, int64_t warm_chunks, float qmax, float sx_mul,
    int tiled)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int K = nb * kBlock;
    const int nw = blockDim.x >> 6;
    const uint2 *const tbl = reinterpret_cast<const uint2 *>(lds_raw);
    constexpr int AMW = ASYM ? 32 : 16;              // floats per wave in the exchange buffer
    float *const amax_s = reinterpret_cast<float *>(lds_raw + diag_table_bytes(nb));   // [2][nw][AMW]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, r = lane & 15;
    const int64_t groups = (M + kTokensPerWG - 1) / kTokensPerWG;

    // The diagonal first: its pieces are staged while the first activations are still in flight.
    // A thread builds whole table entries (block b, element j, lane group g): the four channels
    // 8 (4i + g) + j, i = 0..3, of the block; there are K / 4 entries and at least K / 6 threads,
    // so two rounds cover them.
    const int nent = K >> 2;
    float dv[2][4];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        int e = tid + t * (int)blockDim.x;
        if (e >= nent) e = nent - 1;
        const float *dp = diag + (e >> 5) * kBlock + (e & 3) * 8 + ((e >> 2) & 7);
#pragma unroll
        for (int i = 0; i < 4; ++i) dv[t][i] = diag ? dp[i * 32] : 1.0f;
    }

    // Two raw blocks (64 bytes per lane each) are always in flight: the wave walks the sequence
    // (group, block 0), (group, block 1), ..., (next group, block 0), ... and requests item n + 2
    // into the registers of item n as soon as that one has been unpacked.  Tokens past M are
    // clamped to the last token: they are rotated like the others (every lane takes part in the
    // matrix instructions) and never stored.
    uint4 raw[2][4];
    auto load_raw = [&](uint4 (&dst)[4], int i, int64_t tgl) {
        // unconditional: a block index past the row or a group past the end is clamped to valid
        // memory (a redundant, cached read in the ragged / last step) and its data is not used
        int b = wave + nw * i;                       // wave-uniform
        if (b >= nb) b = nb - 1;
        int64_t token = tgl * kTokensPerWG + r;
        if (token >= M) token = M - 1;
        const uint16_t *src = X + token * ldx + b * kBlock + g * 8;
#pragma unroll
        for (int s = 0; s < 4; ++s) dst[s] = *reinterpret_cast<const uint4 *>(src + s * 32);
    };

    int64_t tg = blockIdx.x;
    load_raw(raw[0], 0, tg);
    if (SPW > 1) load_raw(raw[1], 1, tg);
    else load_raw(raw[1], 0, tg + gridDim.x);
    // the diagonal in three bf16 pieces (truncations: each remainder is exact in fp32)
    {
        uint2 *const tblw = reinterpret_cast<uint2 *>(lds_raw);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int e = tid + t * (int)blockDim.x;
            if (e < nent) {
                uint32_t pc[3][4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float d = dv[t][i];
                    const uint32_t hi = __float_as_uint(d) & 0xFFFF0000u;
                    const float r1 = d - __uint_as_float(hi);
                    const uint32_t mid = __float_as_uint(r1) & 0xFFFF0000u;
                    const uint32_t lo = __float_as_uint(r1 - __uint_as_float(mid));  // at most 8 significant bits
                    pc[0][i] = hi; pc[1][i] = mid; pc[2][i] = lo;
                }
                // entry index ((b * 8 + j) * 3 + piece) * 4 + g with e = (b * 8 + j) * 4 + g
                uint2 *dst = tblw + (size_t)(e >> 2) * 12 + (e & 3);
#pragma unroll
                for (int k = 0; k < 3; ++k)
                    dst[k * 4] = make_uint2(__builtin_amdgcn_perm(pc[k][1], pc[k][0], 0x07060302u),
                                            __builtin_amdgcn_perm(pc[k][3], pc[k][2], 0x07060302u));
            }
        }
    }
    __syncthreads();

    // Row m = 4g' + i of a result lands in lane group g', register i; the row of the A operand
    // that lane r supplies is H_16 row q = pi(r), with pi chosen so that lane group g' receives
    // chunks 2g', 2g'+1 (i = 0, 1) and 8 + 2g', 9 + 2g' (i = 2, 3).
    const int qrow = (r & 2) ? 8 + 2 * (r >> 2) + (r & 1) : 2 * (r >> 2) + (r & 1);
    // sign bits of H_16[qrow][p] for the lane's four p = 4s + g, as bf16 pairs (s = 0, 1 | 2, 3)
    const uint32_t sg0 = ((__builtin_popcount(qrow & g) & 1) ? 0x00008000u : 0u) |
                         ((__builtin_popcount(qrow & (4 + g)) & 1) ? 0x80000000u : 0u);
    const uint32_t sg1 = ((__builtin_popcount(qrow & (8 + g)) & 1) ? 0x00008000u : 0u) |
                         ((__builtin_popcount(qrow & (12 + g)) & 1) ? 0x80000000u : 0u);

    // Optional: read the next kernel's weights once (at most four 16-byte pieces per lane, spread
    // over the whole grid; more than that is left cold).  They only have to pass through the
    // memory-side cache so that the product kernel does not start on cold DRAM: the copies go
    // straight to a 1 KB dump area in LDS that nobody reads, so they hold no registers and nothing
    // waits for them before the end of the kernel.  They are issued after the first token group's
    // rotation, when this wave's own activations have arrived and the memory system is no longer
    // busy with the launch's first wave of loads.  (The compiler does not see them in its count
    // of outstanding loads: its waits can only become stricter by that, never too weak, because
    // the counter retires in order.)
    bool warm_pending = warm_chunks > 0;
    auto issue_warm = [&]() {
        const uint32_t dump = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds_raw +
                              (uint32_t)(diag_table_bytes(nb) + sizeof(float) * 2 * nw * AMW);
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
    };

    int parity = 0;
    // one token group; P = ring slot of its first item
    auto do_group = [&](auto ptag, const int64_t tg) {
        constexpr int P = decltype(ptag)::value;
        const int64_t token = tg * kTokensPerWG + r;
        const bool token_ok = token < M;

        v4f out[SPW][8];   // out[i][j][q']: element j of chunk (q' < 2 ? 2g + q' : 6 + 2g + q') of block wave + nw*i, token r
        float amax = 0.0f;                 // ASYM: the token maximum (>= 0)
        float amin = 0.0f;                 // ASYM: the token minimum (<= 0)
#pragma unroll
        for (int i = 0; i < SPW; ++i) {
            const int b = wave + nw * i;
            if (b < nb) {
                // H_16 with the diagonal folded in, on the matrix pipe: three pieces per j.  The B
                // operand is element j of the four chunks (two bf16 per register, k order s = 0..3).
                const uint4 (&rw)[4] = raw[(P + i) & 1];
                v4f u[8];
                const uint2 *tb = tbl + (size_t)b * (8 * 3 * 4) + g;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
                    const uint32_t w0 = j < 2 ? rw[0].x : j < 4 ? rw[0].y : j < 6 ? rw[0].z : rw[0].w;
                    const uint32_t w1 = j < 2 ? rw[1].x : j < 4 ? rw[1].y : j < 6 ? rw[1].z : rw[1].w;
                    const uint32_t w2 = j < 2 ? rw[2].x : j < 4 ? rw[2].y : j < 6 ? rw[2].z : rw[2].w;
                    const uint32_t w3 = j < 2 ? rw[3].x : j < 4 ? rw[3].y : j < 6 ? rw[3].z : rw[3].w;
                    union { uint32_t w[2]; v4s v; } bop;
                    bop.w[0] = __builtin_amdgcn_perm(w1, w0, sel);
                    bop.w[1] = __builtin_amdgcn_perm(w3, w2, sel);
                    v4f acc = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int pc = 0; pc < 3; ++pc) {
                        const uint2 c = tb[(j * 3 + pc) * 4];
                        union { uint32_t w[2]; v4s v; } aop;
                        aop.w[0] = c.x ^ sg0; aop.w[1] = c.y ^ sg1;
                        acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(aop.v, bop.v, acc, 0, 0, 0);
                    }
                    u[j] = acc;
                }
                // these registers are free: request the item after the next one of the sequence
                load_raw(raw[(P + i) & 1], (i + 2) % SPW, tg + (int64_t)((i + 2) / SPW) * gridDim.x);
                // H_8 over j inside the lane, for each of the four rows
#pragma unroll
                for (int h = 1; h < 8; h <<= 1) {
#pragma unroll
                    for (int j0 = 0; j0 < 8; j0 += 2 * h) {
#pragma unroll
                        for (int j = j0; j < j0 + h; ++j) {
                            const v4f a = u[j], c = u[j + h];
                            u[j] = a + c;
                            u[j + h] = a - c;
                        }
                    }
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    out[i][j] = u[j];
                    if constexpr (ASYM) {
                        amax = fmaxf(fmaxf(amax, u[j][0]), u[j][1]);
                        amax = fmaxf(fmaxf(amax, u[j][2]), u[j][3]);
                        amin = fminf(fminf(amin, u[j][0]), u[j][1]);
                        amin = fminf(fminf(amin, u[j][2]), u[j][3]);
                    } else {
                        amax = fmaxf(fmaxf(amax, fabsf(u[j][0])), fabsf(u[j][1]));     // two v_max3_f32
                        amax = fmaxf(fmaxf(amax, fabsf(u[j][2])), fabsf(u[j][3]));
                    }
                }
            } else {
                // ragged last slot: still advance the sequence
                load_raw(raw[(P + i) & 1], (i + 2) % SPW, tg + (int64_t)((i + 2) / SPW) * gridDim.x);
            }
        }

        if (warm_pending) {
            issue_warm();
            warm_pending = false;
        }

        // token absmax: over the four lane-rows of this wave, then over the waves through LDS
        amax = fmaxf(amax, __shfl_xor(amax, 16));
        amax = fmaxf(amax, __shfl_xor(amax, 32));
        float *const am = amax_s + parity * nw * AMW;
        if (g == 0) am[wave * AMW + r] = amax;
        if constexpr (ASYM) {
            amin = fminf(amin, __shfl_xor(amin, 16));
            amin = fminf(amin, __shfl_xor(amin, 32));
            if (g == 0) am[wave * AMW + 16 + r] = amin;
        }
        __syncthreads();
        for (int wv = 0; wv < nw; ++wv) amax = fmaxf(amax, am[wv * AMW + r]);
        if constexpr (ASYM)
            for (int wv = 0; wv < nw; ++wv) amin = fminf(amin, am[wv * AMW + 16 + r]);
        parity ^= 1;   // the next group writes the other buffer, so one barrier per group suffices

        // out holds sqrt(128) * V.  Symmetric: s_x = max|V| / 127, codes = rint(V / s_x) =
        // rint(out * 127 / max|out|).  Asymmetric (range [lo, hi] with lo <= 0 <= hi): s_x = (hi - lo) / 255,
        // z = -rint(lo / s_x), stored code = clamp(rint(V / s_x) + z, 0, 255) - 128; the integer offset
        // rides in the rounding constant of the same FMA.
        float inv, magic = kRoundMagic;
        if constexpr (ASYM) {
            const float range = amax - amin;
            inv = range > 0.0f ? 255.0f / range : 0.0f;
            const float z = -rintf(amin * inv);                       // 0 .. 255
            magic = kRoundMagic + (z - 128.0f);
            if (wave == 0 && g == 0 && token_ok) {
                sx[token] = range * (0.08838834764831845f / 255.0f);
                zc[token] = 128 - (int)z;
            }
        } else {
            // qmax = 2^(bits-1) - 1 (127 for int8), sx_mul = (1 / sqrt(128)) / qmax, both from the host
            inv = amax > 0.0f ? qmax / amax : 0.0f;
            if (wave == 0 && g == 0 && token_ok) sx[token] = amax * sx_mul;
        }
        // rounded value + offset, clamped to the int8 range, as the low byte of the float's bits
        auto code_bits = [&](float v) -> uint32_t {
            if constexpr (ASYM) {
                const float t = __builtin_fmaf(v, inv, magic);
                return __float_as_uint(__builtin_amdgcn_fmed3f(t, kRoundMagic - 128.0f, kRoundMagic + 127.0f));
            } else {
                return quant_bits(v, inv);
            }
        };

#pragma unroll
        for (int i = 0; i < SPW; ++i) {
            const int b = wave + nw * i;
            if (b < nb && token_ok) {
                uint32_t c[8];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    c[2 * q] = pack4_low_bytes(code_bits(out[i][0][q]), code_bits(out[i][1][q]),
                                               code_bits(out[i][2][q]), code_bits(out[i][3][q]));
                    c[2 * q + 1] = pack4_low_bytes(code_bits(out[i][4][q]), code_bits(out[i][5][q]),
                                                   code_bits(out[i][6][q]), code_bits(out[i][7][q]));
                }
                // row-major: the two 64-byte halves of the block inside the token's row; tiled: piece g of
                // token r in the two 1 KB blocks (16 tokens x 64 k, piece-major) of this 128-block
                int8_t *dst = tiled ? Xq + (tg * (K >> 6) + 2 * b) * (int64_t)1024 + g * 256 + r * 16
                                    : Xq + token * (int64_t)K + b * kBlock + g * 16;
                *reinterpret_cast<uint4 *>(dst) = make_uint4(c[0], c[1], c[2], c[3]);
                *reinterpret_cast<uint4 *>(dst + (tiled ? 1024 : 64)) = make_uint4(c[4], c[5], c[6], c[7]);
            }
        }
    };
    while (tg < groups) {
        do_group(std::integral_constant<int, 0>{}, tg);
        tg += gridDim.x;
        if (tg >= groups) break;
        do_group(std::integral_constant<int, SPW & 1>{}, tg);
        tg += gridDim.x;
    }
    // the copies to the dump area must have landed before the workgroup's LDS is given away
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

template <int SPW, int MAXT>
hipError_t launch_spw(const uint16_t *X, int64_t M, int nb, int nw, int64_t ldx, const float *diag,
                      int8_t *Xq, float *sx, int32_t *zc, const void *warm, int64_t warm_bytes, int wgs_per_cu,
                      hipStream_t st, int abits, bool tiled)
{
    const float qmax = (float)((1 << (abits - 1)) - 1);
    const float sx_mul = 0.08838834764831845f / qmax;
    // persistent workgroups: a few per compute unit, each walking token groups
    const int64_t groups = (M + kTokensPerWG - 1) / kTokensPerWG;
    int64_t grid = (int64_t)num_cus() * wgs_per_cu;
    if (grid > groups) grid = groups;
    const size_t smem = diag_table_bytes(nb) + sizeof(float) * (size_t)2 * nw * (zc ? 32 : 16) + 1024;   // table, extrema, dump area
    const int64_t warm_chunks = (warm && warm_bytes < ((int64_t)1 << 32)) ? warm_bytes / 16 : 0;   // 32-bit byte offsets in the copy
    if (zc)
        hipLaunchKernelGGL((rotate_quant_kernel<SPW, MAXT, true>), dim3((unsigned)grid), dim3(64 * nw), smem, st,
                           X, M, nb, ldx, diag, Xq, sx, zc, static_cast<const uint4 *>(warm), warm_chunks, qmax, sx_mul,
                           (int)tiled);
    else
        hipLaunchKernelGGL((rotate_quant_kernel<SPW, MAXT, false>), dim3((unsigned)grid), dim3(64 * nw), smem, st,
                           X, M, nb, ldx, diag, Xq, sx, zc, static_cast<const uint4 *>(warm), warm_chunks, qmax, sx_mul,
                           (int)tiled);
    return hipGetLastError();
}

}  // namespace

// Largest K: 12 waves x 3 blocks x 128 channels (a workgroup's waves must be co-resident, three
// per SIMD, which leaves 168 registers per lane: room for three blocks of results).
constexpr int kRQMaxBlocks = 36;

hipError_t launch_rotate_quant(const uint16_t *X, int64_t M, int K, int64_t ldx, const float *diag,
                               int8_t *Xq, float *sx, int32_t *zc, const void *warm, int64_t warm_bytes, hipStream_t st,
                               int abits, bool tiled)
{
    if (M == 0) return hipSuccess;
    if (abits < 2 || abits > 8) return hipErrorInvalidValue;
    const int nb = K / kBlock;
    if (nb > kRQMaxBlocks)
        return (zc || abits != 8 || tiled) ? hipErrorInvalidValue : launch_rotate_quant_wide(X, M, K, ldx, diag, Xq, sx, st);
    // three blocks per wave (two or one for narrow rows), then rebalance; workgroups of up to
    // 12 waves, as many per compute unit as stay resident (with three blocks per wave the kernel
    // holds 166 registers and small workgroups pack two waves per SIMD, eight per compute unit)
    int spw = nb < 3 ? nb : 3;
    // few token groups (fewer than six waves per compute unit): spread each row over more waves
    // instead, so that the loads in flight still cover the memory latency
    const int64_t groups = (M + kTokensPerWG - 1) / kTokensPerWG;
    while (spw > 1 && groups * ((nb + spw - 1) / spw) < (int64_t)num_cus() * 6 && (nb + spw - 2) / (spw - 1) <= 12) --spw;
    const int nw = (nb + spw - 1) / spw;
    spw = (nb + nw - 1) / nw;
    const int resident = spw == 3 ? 8 : 12;
    const int wgs = resident / nw > 0 ? resident / nw : 1;
    const bool small = nw <= 4;      // up to 256 threads: no register cap from co-residency
    switch (spw) {
        case 1: return small ? launch_spw<1, 256>(X, M, nb, nw, ldx, diag, Xq, sx, zc, warm, warm_bytes, wgs, st, abits, tiled)
                             : launch_spw<1, 768>(X, M, nb, nw, ldx, diag, Xq, sx, zc, warm, warm_bytes, wgs, st, abits, tiled);
        case 2: return small ? launch_spw<2, 256>(X, M, nb, nw, ldx, diag, Xq, sx, zc, warm, warm_bytes, wgs, st, abits, tiled)
                             : launch_spw<2, 768>(X, M, nb, nw, ldx, diag, Xq, sx, zc, warm, warm_bytes, wgs, st, abits, tiled);
        default: return small ? launch_spw<3, 256>(X, M, nb, nw, ldx, diag, Xq, sx, zc, warm, warm_bytes, wgs, st, abits, tiled)
                              : launch_spw<3, 768>(X, M, nb, nw, ldx, diag, Xq, sx, zc, warm, warm_bytes, wgs, st, abits, tiled);
    }
}

}  // namespace trdq
