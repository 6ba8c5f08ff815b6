// linear_fused: rotate -> per-token quantise -> int8 product -> dequantising epilogue in one
// kernel (Eq. 10 end to end); the int8 activations never leave the chip.
//
// A workgroup owns a panel of BM tokens for the WHOLE input width K: the prologue rotates and
// quantises the panel straight into LDS (int8, BM x K), then the workgroup sweeps its share
// of the output channels with the same matrix-core loop as qgemm, streaming weight tiles
// through a double-buffered LDS stage.  The 160 KB of LDS per compute unit bound BM * K; the
// panel height shrinks as K grows (64 tokens up to K = 1536, 32 up to 3072, 16 up to 6144).
#include <type_traits>

#include "rotate_core.h"

namespace trdq {

namespace {

constexpr int kThreads = 256;
constexpr int kPad = 16;
constexpr int kBN = 128;   // output channels per weight tile
constexpr int kBK = 128;   // input channels per weight tile = one rotation block / scale group
constexpr int64_t kSmallMaxWorkgroups = 512;    // few-token kernel: at most two rounds of workgroups

struct FusedArgs {
    const uint16_t *X;     // bf16 [M, ldx]
    const float *diag;     // [K] or null
    const void *Wc;
    const float *sw;
    const float *bias;
    const int32_t *colsum; // ASYM kernels: sum over k of the weight codes of every output channel [N]
    uint16_t *Y;
    int64_t M, ldx, ldy;
    int K, N;
    int tiles_n;           // ceil(N / kBN)
    int nsplit;            // workgroups sharing one token panel
};

// BM tokens per panel, S lane-rows per token in the prologue, T blocks per lane-row.
// ASYM: the panel is quantised with the asymmetric form of Eq. 1-3 (per-token zero point z, codes
// stored as q - 128); the epilogue adds (128 - z_m) * colsum[n] to the integer sums, which makes
// them the exact sums of (q - z) * w.  Int8 weights only.
template <int BM, int T, int S, bool W4, bool ASYM = false>
__global__ __launch_bounds__(kThreads) void linear_fused_kernel(FusedArgs g)
{
    static_assert(!(W4 && ASYM), "zero points are carried for int8 weights only");
    constexpr int WM = BM >= 64 ? 32 : BM;           // wave tile (tokens)
    constexpr int WGM = BM / WM, WGN = 4 / WGM;
    constexpr int WN = kBN / WGN;
    constexpr int TM = WM / 16, TN = WN / 16;
    constexpr int LDW = kBK + kPad;
    constexpr int CW = W4 ? kBN * (kBK / 32) / kThreads : kBN * (kBK / 16) / kThreads;

    extern __shared__ __align__(16) int8_t smem[];
    const int K = g.K;
    const int nb = K / kBlock;
    const int LDX = K + kPad;
    int8_t *const Xp = smem;                              // [BM][K + 16]   int8 panel
    int8_t *const Ws = smem + BM * LDX;                   // [2][kBN][LDW]  weight stages
    float *const sxs = reinterpret_cast<float *>(Ws + 2 * kBN * LDW);   // [BM]
    int *const zcs = reinterpret_cast<int *>(sxs + BM);                 // [BM] 128 - z (ASYM)

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lg = lane >> 4;
    const int64_t m0 = (int64_t)blockIdx.x * BM;

    // ---- prologue: rotate + quantise the panel into LDS -----------------------------------
    {
        const LaneSigns sg(l16);
        const int s = lg % S;
        constexpr int kTokPerPass = (kThreads / 64) * (4 / S);
        for (int r0 = 0; r0 < BM; r0 += kTokPerPass) {
            const int r = r0 + wave * (4 / S) + lg / S;
            const int64_t token = m0 + r;
            const bool ok = r < BM && token < g.M;
            float v[T][8];
            float amax, amin;
            rotate_token<T, S, ASYM>(g.X + token * g.ldx, ok, nb, s, l16, g.diag, sg, v, amax, amin);
            if constexpr (ASYM) {
                const TokenRangeQuant q(amin, amax);
                if (r < BM) {
                    if (s == 0 && l16 == 0) {
                        sxs[r] = ok ? q.scale : 0.0f;
                        zcs[r] = ok ? q.zc : 0;
                    }
#pragma unroll
                    for (int t = 0; t < T; ++t) {
                        const int b = t * S + s;
                        if (b < nb)
                            *reinterpret_cast<uint2 *>(Xp + r * LDX + b * kBlock + l16 * 8) = q.pack8(v[t]);
                    }
                }
            } else {
                const float inv = token_inv_scale(amax);
                if (r < BM) {
                    if (s == 0 && l16 == 0) sxs[r] = ok ? token_scale(amax) : 0.0f;
#pragma unroll
                    for (int t = 0; t < T; ++t) {
                        const int b = t * S + s;
                        if (b < nb)
                            *reinterpret_cast<uint2 *>(Xp + r * LDX + b * kBlock + l16 * 8) = quant_pack8(v[t], inv);
                    }
                }
            }
        }
    }

    // ---- weight staging -----------------------------------------------------------------------
    const int wm = wave % WGM, wn = wave / WGM;
    const int tiles_per = (g.tiles_n + g.nsplit - 1) / g.nsplit;
    const int tn_begin = blockIdx.y * tiles_per;
    const int tn_end = min(tn_begin + tiles_per, g.tiles_n);
    const int KT = K / kBK;
    const int iters = (tn_end - tn_begin) * KT;

    uint4 wr[CW];
    int wrow[CW], wcol[CW], wdst[CW];
#pragma unroll
    for (int i = 0; i < CW; ++i) {
        const int ch = tid + i * kThreads;
        if constexpr (W4) {
            wrow[i] = ch / (kBK / 32); wcol[i] = (ch % (kBK / 32)) * 16;
            wdst[i] = wrow[i] * LDW + (ch % (kBK / 32)) * 32;
        } else {
            wrow[i] = ch / (kBK / 16); wcol[i] = (ch % (kBK / 16)) * 16;
            wdst[i] = wrow[i] * LDW + wcol[i];
        }
    }
    auto load_tile = [&](int it) {
        const int tn = tn_begin + it / KT, kt = it % KT;
#pragma unroll
        for (int i = 0; i < CW; ++i) {
            int n = tn * kBN + wrow[i];
            if (n >= g.N) n = g.N - 1;
            const uint8_t *src = static_cast<const uint8_t *>(g.Wc) +
                                 (W4 ? (size_t)n * (K / 2) + kt * (kBK / 2) : (size_t)n * K + kt * kBK) + wcol[i];
            wr[i] = *reinterpret_cast<const uint4 *>(src);
        }
    };
    auto store_tile = [&](int buf) {
        int8_t *ws = Ws + buf * kBN * LDW;
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

    v4i acc[TN][TM];
    v4f facc[W4 ? TN : 1][W4 ? TM : 1];
    auto reset = [&]() {
#pragma unroll
        for (int a = 0; a < TN; ++a)
#pragma unroll
            for (int b = 0; b < TM; ++b) {
                acc[a][b] = v4i{0, 0, 0, 0};
                if constexpr (W4) facc[a][b] = v4f{0.f, 0.f, 0.f, 0.f};
            }
    };
    reset();

    if (iters > 0) { load_tile(0); store_tile(0); }
    __syncthreads();     // also publishes the panel and the token scales

    const int8_t *xrow = Xp + (wm * WM + l16) * LDX + lg * 16;
    for (int it = 0; it < iters; ++it) {
        const int buf = it & 1;
        const int tn = tn_begin + it / KT, kt = it % KT;
        if (it + 1 < iters) load_tile(it + 1);

        const int8_t *ws = Ws + buf * kBN * LDW + (wn * WN + l16) * LDW + lg * 16;
#pragma unroll
        for (int kk = 0; kk < kBK; kk += 64) {
            v4i af[TN], bf[TM];
#pragma unroll
            for (int a = 0; a < TN; ++a) af[a] = *reinterpret_cast<const v4i *>(ws + a * 16 * LDW + kk);
#pragma unroll
            for (int b = 0; b < TM; ++b)
                bf[b] = *reinterpret_cast<const v4i *>(xrow + b * 16 * LDX + kt * kBK + kk);
#pragma unroll
            for (int a = 0; a < TN; ++a)
#pragma unroll
                for (int b = 0; b < TM; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[a], bf[b], acc[a][b], 0, 0, 0);
        }

        const int n_base = tn * kBN + wn * WN + lg * 4;
        if constexpr (W4) {
#pragma unroll
            for (int a = 0; a < TN; ++a) {
                const int n = n_base + a * 16;
                float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
                if (n < g.N) s = *reinterpret_cast<const float4 *>(g.sw + (size_t)kt * g.N + n);
#pragma unroll
                for (int b = 0; b < TM; ++b) {
                    facc[a][b][0] += s.x * (float)acc[a][b][0];
                    facc[a][b][1] += s.y * (float)acc[a][b][1];
                    facc[a][b][2] += s.z * (float)acc[a][b][2];
                    facc[a][b][3] += s.w * (float)acc[a][b][3];
                    acc[a][b] = v4i{0, 0, 0, 0};
                }
            }
        }

        if (kt == KT - 1) {
            // epilogue of channel tile tn
#pragma unroll
            for (int a = 0; a < TN; ++a) {
                const int n = n_base + a * 16;
                if (n >= g.N) continue;
                float4 s = make_float4(1.f, 1.f, 1.f, 1.f), bi = make_float4(0.f, 0.f, 0.f, 0.f);
                if constexpr (!W4) s = *reinterpret_cast<const float4 *>(g.sw + n);
                if (g.bias) bi = *reinterpret_cast<const float4 *>(g.bias + n);
                int4 cs = make_int4(0, 0, 0, 0);
                if constexpr (ASYM) cs = *reinterpret_cast<const int4 *>(g.colsum + n);
#pragma unroll
                for (int b = 0; b < TM; ++b) {
                    const int r = wm * WM + b * 16 + l16;
                    const int64_t m = m0 + r;
                    if (m >= g.M) continue;
                    const float sxm = W4 ? sxs[r] * 0.0625f : sxs[r];
                    if constexpr (ASYM) {
                        const int zc = zcs[r];
                        acc[a][b] += v4i{zc * cs.x, zc * cs.y, zc * cs.z, zc * cs.w};
                    }
                    float y0, y1, y2, y3;
                    if constexpr (W4) {
                        y0 = sxm * facc[a][b][0] + bi.x;
                        y1 = sxm * facc[a][b][1] + bi.y;
                        y2 = sxm * facc[a][b][2] + bi.z;
                        y3 = sxm * facc[a][b][3] + bi.w;
                    } else {
                        y0 = (float)acc[a][b][0] * sxm * s.x + bi.x;
                        y1 = (float)acc[a][b][1] * sxm * s.y + bi.y;
                        y2 = (float)acc[a][b][2] * sxm * s.z + bi.z;
                        y3 = (float)acc[a][b][3] * sxm * s.w + bi.w;
                    }
                    uint2 o;
                    o.x = pack_bf16x2(y0, y1);
                    o.y = pack_bf16x2(y2, y3);
                    *reinterpret_cast<uint2 *>(g.Y + m * g.ldy + n) = o;
                }
            }
            reset();
        }

        if (it + 1 < iters) store_tile(buf ^ 1);
        __syncthreads();
    }
}

// ---- few tokens: one 16-token panel per workgroup, K split over eight waves ---------------------
// With a few hundred tokens the unfused pair is bound by two launches and two chains of memory
// latency, not by arithmetic.  Here a workgroup of eight waves owns 16 tokens and BN = 16 * TN
// output channels.  Every weight byte of its slab meets exactly one matrix instruction (there is
// one token tile), so staging weights in LDS would buy nothing: wave w loads the fragments of
// its k-steps (64 input channels each; steps w, w + 8, w + 16) straight from global memory into
// registers, all of them up front, right after the loads of the activations, so that they are
// in flight while the panel is rotated and quantised into LDS.  Then each wave multiplies its
// k-steps, the eight partial sums meet in LDS, and wave w finishes channel tiles w and w + 8.
// K <= 1536 (three k-steps per wave, 108 fragment registers), int8 weights.
constexpr int kSmallThreads = 512;
constexpr int kSmallSteps = 3;

template <int TN, int T, bool ASYM = false>
__global__ __launch_bounds__(kSmallThreads) void linear_fused_small_kernel(FusedArgs g)
{
    constexpr int BN = TN * 16;
    extern __shared__ __align__(16) int8_t smem[];
    const int K = g.K;
    const int nb = K / kBlock;
    const int LDX = K + kPad;
    int8_t *const Xp = smem;                                              // [16][K + 16] int8 panel
    float *const sxs = reinterpret_cast<float *>(smem + 16 * LDX);       // [16]
    int *const zcs = reinterpret_cast<int *>(smem + 16 * LDX + 64);      // [16] 128 - z (ASYM)
    v4i *const part = reinterpret_cast<v4i *>(smem + 16 * LDX + 128);    // [8][TN][64] partial sums
    float *const dl = reinterpret_cast<float *>(part);                   // [K] diagonal (before the sums need the space)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lg = lane >> 4;
    const int tile = blockIdx.x % g.tiles_n, panel = blockIdx.x / g.tiles_n;
    const int64_t m0 = (int64_t)panel * 16;
    const int n0 = tile * BN;
    const int KS = K / 64;

    // Loads return in order, so the order of issue is the order of need: the diagonal (one 16-byte
    // piece per thread, shared through LDS), the activations, then the weight fragments.
    float4 dpiece = make_float4(1.f, 1.f, 1.f, 1.f);
    if (g.diag && tid * 4 < K) dpiece = *reinterpret_cast<const float4 *>(g.diag + tid * 4);
    const int r = wave * 2 + (lg >> 1), s = lg & 1;     // token of this lane row, and which half of its blocks
    const int64_t token = m0 + r;
    const bool tok_ok = token < g.M;
    uint4 raw[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const int b = t * 2 + s;
        raw[t] = make_uint4(0, 0, 0, 0);
        if (tok_ok && b < nb)
            raw[t] = *reinterpret_cast<const uint4 *>(g.X + token * g.ldx + (int64_t)b * kBlock + l16 * 8);
    }

    // this wave's weight fragments: channel n0 + 16a + l16, input channels 64 * step + 16 * lg .. + 15
    v4i wf[kSmallSteps][TN];
    auto load_w = [&](auto ic) {
        constexpr int i = decltype(ic)::value;
        const int step = wave + 8 * i;
        if (step < KS) {
#pragma unroll
            for (int a = 0; a < TN; ++a) {
                int n = n0 + a * 16 + l16;
                if (n >= g.N) n = g.N - 1;
                wf[i][a] = *reinterpret_cast<const v4i *>(static_cast<const int8_t *>(g.Wc) + (size_t)n * K + step * 64 + lg * 16);
            }
        } else {
#pragma unroll
            for (int a = 0; a < TN; ++a) wf[i][a] = v4i{0, 0, 0, 0};
        }
    };
    load_w(std::integral_constant<int, 0>{});
    load_w(std::integral_constant<int, 1>{});
    if (tid * 4 < K) *reinterpret_cast<float4 *>(dl + tid * 4) = dpiece;
    __syncthreads();

    // rotate and quantise the panel into LDS
    {
        const LaneSigns sg(l16);
        float v[T][8];
        float amax = 0.0f, amin = 0.0f;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int b = t * 2 + s < nb ? t * 2 + s : nb - 1;
            const float4 d0 = *reinterpret_cast<const float4 *>(dl + b * kBlock + l16 * 8);
            const float4 d1 = *reinterpret_cast<const float4 *>(dl + b * kBlock + l16 * 8 + 4);
            v[t][0] = bf16_lo(raw[t].x) * d0.x;
            v[t][1] = bf16_hi(raw[t].x) * d0.y;
            v[t][2] = bf16_lo(raw[t].y) * d0.z;
            v[t][3] = bf16_hi(raw[t].y) * d0.w;
            v[t][4] = bf16_lo(raw[t].z) * d1.x;
            v[t][5] = bf16_hi(raw[t].z) * d1.y;
            v[t][6] = bf16_lo(raw[t].w) * d1.z;
            v[t][7] = bf16_hi(raw[t].w) * d1.w;
            fwht128_rows16(v[t], sg);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if constexpr (ASYM) {
                    amax = fmaxf(amax, v[t][j]);
                    amin = fminf(amin, v[t][j]);
                } else {
                    amax = fmaxf(amax, fabsf(v[t][j]));
                }
            }
            if (t == 0) {
                // the last k-step's fragments go out once the first block is done (the queue has drained by then)
                __builtin_amdgcn_sched_barrier(0);
                load_w(std::integral_constant<int, 2>{});
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        amax = row16_max(amax);
        amax = fmaxf(amax, __shfl_xor(amax, 16));
        if constexpr (ASYM) {
            amin = -row16_max(-amin);
            amin = fminf(amin, __shfl_xor(amin, 16));
            const TokenRangeQuant q(amin, amax);
            if (s == 0 && l16 == 0) {
                sxs[r] = tok_ok ? q.scale : 0.0f;
                zcs[r] = tok_ok ? q.zc : 0;
            }
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const int b = t * 2 + s;
                if (b < nb) *reinterpret_cast<uint2 *>(Xp + r * LDX + b * kBlock + l16 * 8) = q.pack8(v[t]);
            }
        } else {
            const float inv = token_inv_scale(amax);
            if (s == 0 && l16 == 0) sxs[r] = tok_ok ? token_scale(amax) : 0.0f;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const int b = t * 2 + s;
                if (b < nb) *reinterpret_cast<uint2 *>(Xp + r * LDX + b * kBlock + l16 * 8) = quant_pack8(v[t], inv);
            }
        }
    }
    __syncthreads();        // panel and scales published; every wave is done with the diagonal

    v4i acc[TN];
#pragma unroll
    for (int a = 0; a < TN; ++a) acc[a] = v4i{0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < kSmallSteps; ++i) {
        const int step = wave + 8 * i;
        if (step < KS) {
            const v4i xf = *reinterpret_cast<const v4i *>(Xp + l16 * LDX + step * 64 + lg * 16);
#pragma unroll
            for (int a = 0; a < TN; ++a)
                acc[a] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[i][a], xf, acc[a], 0, 0, 0);
        }
    }
#pragma unroll
    for (int a = 0; a < TN; ++a) part[(wave * TN + a) * 64 + lane] = acc[a];
    __syncthreads();

    // wave w finishes channel tiles w, w + 8: lane holds channels n .. n + 3 of token m0 + l16
    for (int a = wave; a < TN; a += 8) {
        v4i sum = part[a * 64 + lane];
#pragma unroll
        for (int w = 1; w < 8; ++w) sum += part[(w * TN + a) * 64 + lane];
        const int n = n0 + a * 16 + lg * 4;
        const int64_t m = m0 + l16;
        if (n < g.N && m < g.M) {
            const float4 sw = *reinterpret_cast<const float4 *>(g.sw + n);
            float4 bi = make_float4(0.f, 0.f, 0.f, 0.f);
            if (g.bias) bi = *reinterpret_cast<const float4 *>(g.bias + n);
            const float sxm = sxs[l16];
            if constexpr (ASYM) {
                const int4 cs = *reinterpret_cast<const int4 *>(g.colsum + n);
                const int zc = zcs[l16];
                sum += v4i{zc * cs.x, zc * cs.y, zc * cs.z, zc * cs.w};
            }
            uint2 o;
            o.x = pack_bf16x2((float)sum[0] * sxm * sw.x + bi.x, (float)sum[1] * sxm * sw.y + bi.y);
            o.y = pack_bf16x2((float)sum[2] * sxm * sw.z + bi.z, (float)sum[3] * sxm * sw.w + bi.w);
            *reinterpret_cast<uint2 *>(g.Y + m * g.ldy + n) = o;
        }
    }
}

template <int TN, int T, bool ASYM>
hipError_t launch_small(const FusedArgs &a, hipStream_t st)
{
    FusedArgs g = a;
    const int64_t panels = (g.M + 15) / 16;
    g.tiles_n = (g.N + TN * 16 - 1) / (TN * 16);
    const size_t smem = (size_t)16 * (g.K + kPad) + 128 + (size_t)8 * TN * 1024;
    auto kern = linear_fused_small_kernel<TN, T, ASYM>;
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), smem); e != hipSuccess) return e;
    // consecutive workgroups take the channel tiles of one panel: with eight tiles (1152 = 8 x 144)
    // each of the eight dies keeps seeing the same weight slab
    hipLaunchKernelGGL(kern, dim3((unsigned)(panels * g.tiles_n)), dim3(kSmallThreads), smem, st, g);
    return hipGetLastError();
}

// few-token kernel: int8 weights, K <= 1536, and few enough workgroups that repeating the
// rotation per channel tile costs less than a second launch
bool small_applies(const FusedArgs &a, int wbits)
{
    if (wbits != 8 || a.K > 1536) return false;
    const int bn = a.N % 144 == 0 ? 144 : 128;
    const int64_t wgs = ((a.M + 15) / 16) * ((a.N + bn - 1) / bn);
    return wgs <= kSmallMaxWorkgroups;
}

template <int TN, bool ASYM>
hipError_t launch_small_tn(const FusedArgs &a, hipStream_t st)
{
    switch ((a.K / kBlock + 1) / 2) {       // blocks per lane row (two lane rows share a token)
        case 1: return launch_small<TN, 1, ASYM>(a, st);
        case 2: return launch_small<TN, 2, ASYM>(a, st);
        case 3: return launch_small<TN, 3, ASYM>(a, st);
        case 4: return launch_small<TN, 4, ASYM>(a, st);
        case 5: return launch_small<TN, 5, ASYM>(a, st);
        default: return launch_small<TN, 6, ASYM>(a, st);
    }
}

template <bool ASYM>
hipError_t launch_small_any(const FusedArgs &a, hipStream_t st)
{
    return a.N % 144 == 0 ? launch_small_tn<9, ASYM>(a, st) : launch_small_tn<8, ASYM>(a, st);
}

template <int BM, int T, int S, bool W4, bool ASYM>
hipError_t launch_one(const FusedArgs &a, hipStream_t st)
{
    FusedArgs g = a;
    const int64_t panels = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + kBN - 1) / kBN;
    // enough workgroups to fill the compute units twice; every extra split repeats the prologue
    int64_t want = (2 * num_cus() + panels - 1) / panels;
    want = want < 1 ? 1 : (want > g.tiles_n ? g.tiles_n : want);
    const int tiles_per = (int)((g.tiles_n + want - 1) / want);
    g.nsplit = (g.tiles_n + tiles_per - 1) / tiles_per;   // no workgroup without a channel tile
    const size_t smem = (size_t)BM * (g.K + kPad) + 2 * (size_t)kBN * (kBK + kPad) + 2 * BM * sizeof(float);
    auto kern = linear_fused_kernel<BM, T, S, W4, ASYM>;
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), smem); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)panels, (unsigned)g.nsplit), dim3(kThreads), smem, st, g);
    return hipGetLastError();
}

template <int BM, int S, bool W4, bool ASYM>
hipError_t launch_t(int T, const FusedArgs &a, hipStream_t st)
{
    if (T <= 3) return launch_one<BM, 3, S, W4, ASYM>(a, st);
    if (T <= 6) return launch_one<BM, 6, S, W4, ASYM>(a, st);
    if (T <= 9) return launch_one<BM, 9, S, W4, ASYM>(a, st);
    return launch_one<BM, 12, S, W4, ASYM>(a, st);
}

template <bool W4, bool ASYM = false>
hipError_t launch_w(const FusedArgs &a, hipStream_t st)
{
    const int nb = a.K / kBlock;
    if (nb <= 12) return launch_t<64, 1, W4, ASYM>(nb, a, st);
    if (nb <= 24) return launch_t<32, 2, W4, ASYM>((nb + 1) / 2, a, st);
    return launch_t<16, 4, W4, ASYM>((nb + 3) / 4, a, st);
}

}  // namespace

bool fused_supports(int K) { return K % kBlock == 0 && K / kBlock <= 48; }

// True where the fused kernel is the faster path: the few-token kernel in a single round of
// workgroups (measured on 1152-wide layers: 10-11.5 us against 14-15 us for the pair up to 512 tokens).
bool fused_pays(int64_t M, int K, int N, int wbits)
{
    if (wbits != 8 || K > 1536 || K % kBlock != 0 || M <= 0) return false;
    const int bn = N % 144 == 0 ? 144 : 128;
    return ((M + 15) / 16) * ((N + bn - 1) / bn) <= num_cus();
}

hipError_t launch_linear_fused(const Weights &w, const uint16_t *X, int64_t M, int64_t ldx,
                               const float *diag, const float *bias, uint16_t *Y, int64_t ldy,
                               hipStream_t st, bool asym)
{
    if (M == 0) return hipSuccess;
    if (asym && (w.wbits != 8 || !w.colsum)) return hipErrorInvalidValue;
    FusedArgs a;
    a.X = X; a.diag = diag; a.Wc = w.codes; a.sw = w.scales; a.bias = bias; a.colsum = w.colsum; a.Y = Y;
    a.M = M; a.ldx = ldx; a.ldy = ldy; a.K = w.K; a.N = w.N; a.tiles_n = 0; a.nsplit = 1;
    if (small_applies(a, w.wbits)) return asym ? launch_small_any<true>(a, st) : launch_small_any<false>(a, st);
    if (asym) return launch_w<false, true>(a, st);
    return w.wbits == 4 ? launch_w<true>(a, st) : launch_w<false>(a, st);
}

}  // namespace trdq
