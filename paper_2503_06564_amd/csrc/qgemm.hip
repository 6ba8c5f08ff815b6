// qgemm: the integer product G_t(X_t) . H_t(W) of Eq. 10 on the quantised codes, on the
// gfx950 int8 matrix cores (v_mfma_i32_16x16x64_i8, int32 accumulation), with the
// dequantising epilogue (undo the scales of Eq. 1, add the bias, round to bf16).
//
// Operand roles.  The matrix instruction computes D[i][j] = sum_k A[i][k] B[k][j] and leaves
// four consecutive i of one j in each lane.  The weights take the A role (i = output
// channel n) and the activations the B role (j = token m), so every lane ends up with four
// consecutive output channels of one token: one 8-byte bf16 store per 16x16 tile.  Both
// operands are K-contiguous in memory (activations [M, K], prepared weights [N, K]), so both
// are staged the same way: 16-byte chunks through registers into LDS rows padded by 16 bytes,
// read back as 16 bytes per lane (row = lane % 16, k-offset = 16 * (lane / 16)).
//
// int4 weights are widened to int8 while they are copied into LDS, as 16 * code (the nibble
// moved to the top of the byte), so the main loop is the same; at every 128-channel group
// boundary the int32 partial sums are folded into float accumulators with the group's scale.
#include "gemm_common.h"

namespace trdq {

using namespace gemm;

namespace {

constexpr int kPad = 16;  // bytes of padding per LDS row

template <int BM, int BN, int BK, int WGM, int WGN, bool W4, bool DEBUG>
__global__ __launch_bounds__(kThreads) void qgemm_kernel(GemmArgs g)
{
    static_assert(WGM * WGN == 4, "four waves per workgroup");
    static_assert(!W4 || BK == kBlock, "int4: one scale group per k-tile");
    constexpr int WM = BM / WGM, WN = BN / WGN;      // wave tile
    constexpr int TM = WM / 16, TN = WN / 16;        // 16x16 tiles per wave
    constexpr int LDR = BK + kPad;                   // LDS row stride in bytes
    constexpr int CPR = BK / 16;                     // 16-byte chunks per tile row
    constexpr int CX = BM * CPR / kThreads;          // activation chunks per thread
    constexpr int CW = W4 ? BN * (BK / 32) / kThreads : BN * CPR / kThreads;  // weight chunks per thread
    static_assert(CX >= 1 && CW >= 1, "tile too small for 256 threads");

    extern __shared__ __align__(16) int8_t smem[];
    int8_t *const Xs = smem;                         // [2][BM][LDR]
    int8_t *const Ws = smem + 2 * BM * LDR;          // [2][BN][LDR]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WGM, wn = wave / WGM;
    const int l16 = lane & 15, lg = lane >> 4;

    const int tile = xcd_remap(blockIdx.x, g.tiles_m * g.tiles_n);
    const int tm_idx = tile / g.tiles_n, tn_idx = tile % g.tiles_n;
    const int64_t m0 = (int64_t)tm_idx * BM;
    const int n0 = tn_idx * BN;
    const int K = g.K;

    // ---- global -> register staging --------------------------------------------------
    uint4 xr[CX], wr[CW];
    const int8_t *xsrc[CX];
    const uint8_t *wsrc[CW];
    int xdst[CX], wdst[CW];
#pragma unroll
    for (int i = 0; i < CX; ++i) {
        const int ch = tid + i * kThreads;
        const int row = ch / CPR, c16 = ch % CPR;
        int64_t m = m0 + row;
        if (m >= g.M) m = g.M - 1;                    // clamp: rows past M are never stored
        xsrc[i] = g.Xq + m * K + c16 * 16;
        xdst[i] = row * LDR + c16 * 16;
    }
#pragma unroll
    for (int i = 0; i < CW; ++i) {
        const int ch = tid + i * kThreads;
        if constexpr (W4) {
            constexpr int CPR4 = BK / 32;             // 16 packed bytes = 32 channels
            const int row = ch / CPR4, c32 = ch % CPR4;
            int n = n0 + row;
            if (n >= g.N) n = g.N - 1;
            wsrc[i] = static_cast<const uint8_t *>(g.Wc) + (size_t)n * (K / 2) + c32 * 16;
            wdst[i] = row * LDR + c32 * 32;
        } else {
            const int row = ch / CPR, c16 = ch % CPR;
            int n = n0 + row;
            if (n >= g.N) n = g.N - 1;
            wsrc[i] = static_cast<const uint8_t *>(g.Wc) + (size_t)n * K + c16 * 16;
            wdst[i] = row * LDR + c16 * 16;
        }
    }
    auto load_tile = [&](int kt) {
#pragma unroll
        for (int i = 0; i < CX; ++i) xr[i] = *reinterpret_cast<const uint4 *>(xsrc[i] + kt * BK);
#pragma unroll
        for (int i = 0; i < CW; ++i)
            wr[i] = *reinterpret_cast<const uint4 *>(wsrc[i] + (W4 ? kt * (BK / 2) : kt * BK));
    };
    auto store_tile = [&](int buf) {
        int8_t *xs = Xs + buf * BM * LDR, *ws = Ws + buf * BN * LDR;
#pragma unroll
        for (int i = 0; i < CX; ++i) *reinterpret_cast<uint4 *>(xs + xdst[i]) = xr[i];
#pragma unroll
        for (int i = 0; i < CW; ++i) {
            if constexpr (W4) {
                const uint4 p = wr[i];
                uint4 a, b;
                a.x = (p.x << 4) & 0xF0F0F0F0u; a.y = p.x & 0xF0F0F0F0u;
                a.z = (p.y << 4) & 0xF0F0F0F0u; a.w = p.y & 0xF0F0F0F0u;
                b.x = (p.z << 4) & 0xF0F0F0F0u; b.y = p.z & 0xF0F0F0F0u;
                b.z = (p.w << 4) & 0xF0F0F0F0u; b.w = p.w & 0xF0F0F0F0u;
                *reinterpret_cast<uint4 *>(ws + wdst[i]) = a;
                *reinterpret_cast<uint4 *>(ws + wdst[i] + 16) = b;
            } else {
                *reinterpret_cast<uint4 *>(ws + wdst[i]) = wr[i];
            }
        }
    };

    // ---- accumulators ------------------------------------------------------------------
    v4i acc[TN][TM];
    v4f facc[W4 ? TN : 1][W4 ? TM : 1];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b) acc[a][b] = v4i{0, 0, 0, 0};
    if constexpr (W4) {
#pragma unroll
        for (int a = 0; a < TN; ++a)
#pragma unroll
            for (int b = 0; b < TM; ++b) facc[a][b] = v4f{0.f, 0.f, 0.f, 0.f};
    }

    // lane's output coordinates: channels n_lane(a) .. +3, token m_lane(b)
    auto n_lane = [&](int a) { return n0 + wn * WN + a * 16 + lg * 4; };
    auto m_lane = [&](int b) { return m0 + wm * WM + b * 16 + l16; };

    const int KT = K / BK;
    load_tile(0);
    store_tile(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) load_tile(kt + 1);

        const int8_t *xs = Xs + buf * BM * LDR + (wm * WM + l16) * LDR + lg * 16;
        const int8_t *ws = Ws + buf * BN * LDR + (wn * WN + l16) * LDR + lg * 16;
#pragma unroll
        for (int kk = 0; kk < BK; kk += 64) {
            v4i af[TN], bf[TM];
#pragma unroll
            for (int a = 0; a < TN; ++a) af[a] = *reinterpret_cast<const v4i *>(ws + a * 16 * LDR + kk);
#pragma unroll
            for (int b = 0; b < TM; ++b) bf[b] = *reinterpret_cast<const v4i *>(xs + b * 16 * LDR + kk);
#pragma unroll
            for (int a = 0; a < TN; ++a)
#pragma unroll
                for (int b = 0; b < TM; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[a], bf[b], acc[a][b], 0, 0, 0);
        }

        if constexpr (W4) {
            // end of scale group kt: fold 16 * acc_g into the float accumulators
#pragma unroll
            for (int a = 0; a < TN; ++a) {
                const int n = n_lane(a);
                float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
                if (n < g.N) s = *reinterpret_cast<const float4 *>(g.sw + (size_t)kt * g.N + n);
#pragma unroll
                for (int b = 0; b < TM; ++b) {
                    if constexpr (DEBUG) {
                        const int64_t m = m_lane(b);
                        if (m < g.M && n < g.N) {
                            int4 o = make_int4(acc[a][b][0] >> 4, acc[a][b][1] >> 4,
                                               acc[a][b][2] >> 4, acc[a][b][3] >> 4);
                            *reinterpret_cast<int4 *>(g.acc_debug + ((int64_t)kt * g.M + m) * g.N + n) = o;
                        }
                    }
                    facc[a][b][0] += s.x * (float)acc[a][b][0];
                    facc[a][b][1] += s.y * (float)acc[a][b][1];
                    facc[a][b][2] += s.z * (float)acc[a][b][2];
                    facc[a][b][3] += s.w * (float)acc[a][b][3];
                    acc[a][b] = v4i{0, 0, 0, 0};
                }
            }
        }

        if (kt + 1 < KT) store_tile(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue ----------------------------------------------------------------------
    float sxm[TM];
#pragma unroll
    for (int b = 0; b < TM; ++b) {
        const int64_t m = m_lane(b);
        sxm[b] = m < g.M ? g.sx[m] : 0.0f;
        if constexpr (W4) sxm[b] *= 0.0625f;         // the codes were staged as 16 * code
    }
#pragma unroll
    for (int a = 0; a < TN; ++a) {
        const int n = n_lane(a);
        if (n >= g.N) continue;
        float4 s = make_float4(1.f, 1.f, 1.f, 1.f), bi = make_float4(0.f, 0.f, 0.f, 0.f);
        if constexpr (!W4) s = *reinterpret_cast<const float4 *>(g.sw + n);
        if (g.bias) bi = *reinterpret_cast<const float4 *>(g.bias + n);
#pragma unroll
        for (int b = 0; b < TM; ++b) {
            const int64_t m = m_lane(b);
            if (m >= g.M) continue;
            float y0, y1, y2, y3;
            if constexpr (W4) {
                y0 = sxm[b] * facc[a][b][0] + bi.x;
                y1 = sxm[b] * facc[a][b][1] + bi.y;
                y2 = sxm[b] * facc[a][b][2] + bi.z;
                y3 = sxm[b] * facc[a][b][3] + bi.w;
            } else {
                if constexpr (DEBUG) {
                    int4 o = make_int4(acc[a][b][0], acc[a][b][1], acc[a][b][2], acc[a][b][3]);
                    *reinterpret_cast<int4 *>(g.acc_debug + m * g.N + n) = o;
                }
                y0 = (float)acc[a][b][0] * sxm[b] * s.x + bi.x;
                y1 = (float)acc[a][b][1] * sxm[b] * s.y + bi.y;
                y2 = (float)acc[a][b][2] * sxm[b] * s.z + bi.z;
                y3 = (float)acc[a][b][3] * sxm[b] * s.w + bi.w;
            }
            uint2 o;
            o.x = pack_bf16x2(y0, y1);
            o.y = pack_bf16x2(y2, y3);
            *reinterpret_cast<uint2 *>(g.Y + m * g.ldy + n) = o;
        }
    }
}

template <int BM, int BN, int BK, int WGM, int WGN, bool W4>
hipError_t launch_cfg(const GemmArgs &a, bool debug, hipStream_t st)
{
    GemmArgs g = a;
    g.tiles_m = (int)((g.M + BM - 1) / BM);
    g.tiles_n = (g.N + BN - 1) / BN;
    const size_t smem = 2 * (size_t)(BM + BN) * (BK + kPad);
    const dim3 grid((unsigned)(g.tiles_m * g.tiles_n));
    auto kern = debug ? qgemm_kernel<BM, BN, BK, WGM, WGN, W4, true>
                      : qgemm_kernel<BM, BN, BK, WGM, WGN, W4, false>;
    if (smem > 64 * 1024)
        if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), smem); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, dim3(kThreads), smem, st, g);
    return hipGetLastError();
}

}  // namespace

// Tile variants.  0-5: register-staged double buffer {BM, BN, BK} (also the int4 path):
//   0: 128x128x64   1: 128x128x128   2: 256x128x64   3: 128x256x64   4: 256x128x128   5: 64x128x128
// 6 and up: the direct-to-LDS int8 kernels of qgemm_dma.hip (variant - 6 indexes its table).
constexpr int kRegVariants = 6;
int qgemm_num_variants() { return kRegVariants + dma_num_variants() + 1; }

hipError_t launch_qgemm(const Weights &w, const int8_t *Xq, const float *sx, const int32_t *zc, int64_t M,
                        const float *bias, uint16_t *Y, int64_t ldy, int32_t *acc_debug,
                        int variant, hipStream_t st, const int32_t *rowsum)
{
    if (M == 0) return hipSuccess;
    if (w.zcw) {
        // asymmetric weights (int8, per output channel): zero-point terms on both sides in the epilogue of
        // the kernel that takes any shape
        if (w.wbits != 8 || !w.colsum || !rowsum) return hipErrorInvalidValue;
        GemmArgs a;
        a.Xq = Xq; a.Wc = w.codes; a.sx = sx; a.sw = w.scales; a.bias = bias; a.Y = Y;
        a.acc_debug = acc_debug; a.M = M; a.ldy = ldy; a.K = w.K; a.N = w.N;
        a.tiles_m = a.tiles_n = 0;
        a.zc = zc; a.colsum = w.colsum; a.zcw = w.zcw; a.rowsum = rowsum;
        return launch_qgemm8_asym(a, acc_debug != nullptr, 0, st);
    }
    // A ragged token count would send the whole product to the kernel that takes any shape.  With the
    // built-in choice and int8 weights, the whole 256-token (or 128-token) panels go to the fast kernels
    // and only the remaining rows to that kernel, as a second launch on the same stream.
    if (variant < 0 && w.wbits == 8 && M >= 1024 && M % 128 != 0) {
        const int64_t head = M - M % (M % 256 < 128 ? 256 : 128);
        hipError_t e = launch_qgemm(w, Xq, sx, zc, head, bias, Y, ldy, acc_debug, variant, st);
        if (e != hipSuccess) return e;
        return launch_qgemm(w, Xq + head * w.K, sx + head, zc ? zc + head : nullptr, M - head, bias, Y + head * ldy, ldy,
                            acc_debug ? acc_debug + head * w.N : nullptr, variant, st);
    }
    GemmArgs a;
    a.Xq = Xq; a.Wc = w.codes; a.sx = sx; a.sw = w.scales; a.bias = bias; a.Y = Y;
    a.acc_debug = acc_debug; a.M = M; a.ldy = ldy; a.K = w.K; a.N = w.N;
    a.tiles_m = a.tiles_n = 0;
    const bool dbg = acc_debug != nullptr;
    if (zc && w.wbits == 4) {
        // asymmetric activations against int4 weights: the scaled zero-point term is one multiply-add per
        // output in the epilogue of the int4 kernel
        if (!w.colsumw) return hipErrorInvalidValue;
        a.zc = zc;
        a.colsumw = w.colsumw;
        return launch_qgemm4_dma(a, dbg, 0, st);
    }
    if (zc) {
        // asymmetric activations: int8 weights with their column sums; the 128 x 144 kernels where
        // the symmetric path would take them or the 256 x 256 kernel, else the ring kernel
        if (w.wbits != 8 || !w.colsum) return hipErrorInvalidValue;
        a.zc = zc;
        a.colsum = w.colsum;
        int kind = 0;
        if (a.N % 144 == 0 && M % 128 == 0 && a.K >= 512 && ldy % 8 == 0 && reinterpret_cast<uintptr_t>(Y) % 16 == 0) {
            const int64_t tiles144 = (M / 128) * (a.N / 144);
            kind = tiles144 > num_cus() ? 15 : (a.K >= 2304 ? 18 : 14);
        }
        if (variant >= 0) kind = variant;     // tests: 0, 14, 15 or 18
        return launch_qgemm8_asym(a, dbg, kind, st);
    }
    // the row-wise epilogues store 16 bytes per lane: an output whose rows are only 8-byte aligned
    // goes to the kernels that store 8 bytes per lane
    if (ldy % 8 != 0 || reinterpret_cast<uintptr_t>(Y) % 16 != 0)
        return w.wbits == 4 ? launch_cfg<128, 128, 128, 2, 2, true>(a, dbg, st) : launch_qgemm8_dma(a, dbg, 0, st);
    if (w.wbits == 4) {
        // int4 keeps a second (float) accumulator set: smaller tiles, BK = one scale group
        // variants 1 and 5: register-staged; 6, 7: direct-to-LDS (6 is the built-in choice)
        switch (variant) {
            case 1: return launch_cfg<128, 128, 128, 2, 2, true>(a, dbg, st);
            case 5: return launch_cfg<64, 128, 128, 1, 4, true>(a, dbg, st);
            case 7: return launch_qgemm4_dma(a, dbg, 1, st);
            default: return launch_qgemm4_dma(a, dbg, 0, st);
        }
    }
    // built-in choice (measured crossovers on the DiT-XL/2 widths): the 256 x 256 kernel once
    // there are well over 256 of its tiles; below that, where the width is a multiple of 144
    // (1152 = 8 x 144, so whole rounds of tiles), 128 x 144 tiles: at most one tile per compute
    // unit -> one workgroup per compute unit with a four-stage ring, or for long K the kernel whose
    // two wave groups split K inside the workgroup; more tiles -> two stages and two workgroups
    // per compute unit; other widths take the software-pipelined 128 x 128
    // kernel, two workgroups per compute unit (it hands ragged shapes to the ring kernel itself)
    if (variant < 0) {
        variant = kRegVariants + 9;
        const int64_t tiles144 = (a.N % 144 == 0 && M % 128 == 0 && a.K >= 512) ? (M / 128) * (a.N / 144) : 0;
        const int64_t tiles256 = ((M + 255) / 256) * ((a.N + 255) / 256);
        if (tiles144 > 0 && tiles144 <= num_cus())
            variant = a.K >= 2304 ? kRegVariants + 18 : kRegVariants + 14;
        else if (tiles256 >= 400 && wide_supports(a))
            variant = kRegVariants + dma_num_variants();
        else if (tiles144 > 0)
            variant = kRegVariants + 15;
    }
    switch (variant) {
        case 0: return launch_cfg<128, 128, 64, 2, 2, false>(a, dbg, st);
        case 1: return launch_cfg<128, 128, 128, 2, 2, false>(a, dbg, st);
        case 2: return launch_cfg<256, 128, 64, 2, 2, false>(a, dbg, st);
        case 3: return launch_cfg<128, 256, 64, 2, 2, false>(a, dbg, st);
        case 4: return launch_cfg<256, 128, 128, 2, 2, false>(a, dbg, st);
        case 5: return launch_cfg<64, 128, 128, 1, 4, false>(a, dbg, st);
        default:
            // last variant: 256 x 256 tiles, hand-scheduled loop; shapes it does not take go to the
            // ring kernel
            if (variant == kRegVariants + dma_num_variants())
                return wide_supports(a) ? launch_qgemm8_wide(a, dbg, st) : launch_qgemm8_dma(a, dbg, 0, st);
            return launch_qgemm8_dma(a, dbg, variant - kRegVariants, st);
    }
}

bool qgemm_tiled_supports(const Weights &w, int64_t M, const void *Y, int64_t ldy)
{
    if (!w.codes_tiled || (w.wbits != 8 && w.wbits != 4)) return false;
    GemmArgs a;
    a.Xq = nullptr; a.Wc = w.codes_tiled; a.sx = nullptr; a.sw = w.scales; a.bias = nullptr;
    a.Y = static_cast<uint16_t *>(const_cast<void *>(Y)); a.acc_debug = nullptr; a.M = M; a.ldy = ldy; a.K = w.K; a.N = w.N;
    a.tiles_m = a.tiles_n = 0;
    return w.wbits == 4 ? tiled4_supports(a) : tiled_supports(a);
}

hipError_t launch_qgemm_tiled(const Weights &w, const int8_t *Xt, const float *sx, int64_t M, const float *bias,
                              uint16_t *Y, int64_t ldy, int32_t *acc_debug, hipStream_t st)
{
    if (M == 0) return hipSuccess;
    if (!qgemm_tiled_supports(w, M, Y, ldy)) return hipErrorInvalidValue;
    GemmArgs a;
    a.Xq = Xt; a.Wc = w.codes_tiled; a.sx = sx; a.sw = w.scales; a.bias = bias; a.Y = Y;
    a.acc_debug = acc_debug; a.M = M; a.ldy = ldy; a.K = w.K; a.N = w.N;
    a.tiles_m = a.tiles_n = 0;
    return w.wbits == 4 ? launch_qgemm4_tiled(a, acc_debug != nullptr, st) : launch_qgemm8_tiled(a, acc_debug != nullptr, st);
}

bool qgemm_tiled_pays(int64_t M, int K, int N)
{
    // Measured on the DiT-XL/2 widths at 256 ... 32768 tokens.  Up to one 128 x 144 tile per compute
    // unit the kernel that splits K between two wave pairs wins for K >= 1024 (by 5 % at K = 1152, 15-20 %
    // at K = 4608); with more tiles the kernel with two workgroups per compute unit does, by 5-30 %,
    // except for long K at up to two tiles per compute unit, where the row-major kernel whose wave groups
    // split K is level with it.
    const int64_t tiles = (M / 128) * (int64_t)(N / 144);
    if (tiles <= num_cus()) return K >= 1024;
    return !(K >= 2304 && tiles <= 2 * (int64_t)num_cus());
}

hipError_t launch_retile_w4_codes(const void *src, void *dst, int64_t N, int K, hipStream_t st)
{
    return launch_retile_w4(src, dst, N, K, st);
}

hipError_t launch_retile_rows(const int8_t *src, int8_t *dst, int64_t R, int K, bool to_tiled, hipStream_t st)
{
    return launch_retile(src, dst, R, K, to_tiled, st);
}

}  // namespace trdq
