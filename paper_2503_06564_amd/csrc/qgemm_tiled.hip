// W8A8 integer product on block-tiled operands: 256 x 144 (and 128 x 144) output tiles, two
// workgroups per compute unit.
//
// Operation: Y = dequant(Xq . Wq^T) of Eq. 10's quantised product (per-token and per-channel
// scales, optional bias, bf16 output), the arithmetic of the other int8 kernels.
//
// Why another kernel.  With 128 x 144 tiles the k-loop is bound by what the L2 delivers into LDS
// (17 KB of copies per 72 matrix instructions) and by LDS reads (a wave tile of 32 x 144 reads
// 0.6 KB per matrix instruction).  A wave tile of 64 tokens x 144 channels needs 0.36 KB of reads
// and, as a 256 x 144 workgroup tile, 25 KB of copies per 144 matrix instructions.  Two such
// workgroups fit a compute unit only if a k-step is 64 bytes deep (three stages of 25 KB each),
// and a 64-byte-deep copy of row-major operands fetches half cache lines, which doubles the
// traffic between L2 and L1.  Hence both operands are stored in 1 KB blocks of 16 rows x 64 bytes
// of k (block (row / 16, k / 64) at ((row / 16) * K / 64 + k / 64) * 1024, rows 64 bytes apart):
// one direct-to-LDS copy moves one block, eight whole cache lines, and one block is one operand
// fragment of v_mfma_i32_16x16x64_i8.  trdq_rotate_quant_tiled writes activations in this form;
// the weights get a second copy of their codes in it when they are prepared.
//
// A launch may mix tile heights: workgroups [0, n_big) take 256-token tiles over the first nbn
// channel tiles, the others 128-token tiles over the remaining channel tiles, so that a shape
// whose 256-token tiles would fill the chip one and a half times still runs as one round of two
// workgroups per compute unit (a tall and a short one, whose prologues and epilogues fall at
// different times).
#include <type_traits>
#include <utility>

#include "gemm_common.h"

namespace trdq {
namespace gemm {

namespace {

constexpr int kBN = 144;                     // channels per tile
constexpr int kTN = kBN / 16;                // weight fragments per k-step
#ifndef TRDQ_X_NS
#define TRDQ_X_NS 3
#endif
constexpr int kNS = TRDQ_X_NS;               // stages of the ring
constexpr int kStageBig = (256 / 16 + kTN) * 1024;
constexpr int kParOff = 3 * kStageBig;     // epilogue operands: [144 s_w][pad][144 bias][pad][256 s_x]
constexpr int kParSw = 0, kParBias = 1024, kParSx = 2048;
constexpr int kTiledLds = kParOff + 3072;    // 79872 B: two workgroups per compute unit

template <int... Is, class F>
__device__ __forceinline__ void static_for_seq(std::integer_sequence<int, Is...>, F &&f)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for_n(F &&f)
{
    static_for_seq(std::make_integer_sequence<int, N>{}, f);
}

// 16-byte piece p of row r of a block sits at r * 64 + ((p ^ swizzle(r)) * 16) in LDS
__device__ __forceinline__ int blk_off(int r, int p) { return r * 64 + ((p ^ chunk_swizzle<64>(r)) * 16); }

__device__ __forceinline__ void copy_1k_if(int on, uint32_t voff, const void *sbase, uint32_t lds_addr)
{
    asm volatile("s_cmp_eq_u32 %3, 0\n\ts_cbranch_scc1 .Lskip%=\n\t"
                 "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n"
                 ".Lskip%=:"
                 :: "v"(voff), "s"(sbase), "s"(lds_addr), "s"(__builtin_amdgcn_readfirstlane(on))
                 : "memory", "scc");
}

// One output tile of BM tokens x 144 channels.  Wave w owns token rows w * BM/4 .. of the tile
// and all 144 channels: TM = BM / 64 activation fragments (its own, which only it reads) and the
// nine weight fragments (shared) per k-step; the lane ends with channels n .. n+3 of one token per
// accumulator tile.  Per k-step: wait until the next step's blocks have landed, barrier (which
// also retires every read of the current step's stage), refill that stage with the step three
// ahead, then 9 x TM matrix instructions on the fragments in registers while the next step's
// fragments are read: a weight fragment's registers are refilled as soon as its TM instructions
// have issued, the activation fragments alternate between two sets.
template <int BM, bool DEBUG>
__device__ __forceinline__ void run_tile(const GemmArgs &g, int tm, int tn, int8_t *smem)
{
    constexpr int TM = BM / 64;
    constexpr int XB = BM / 16;                       // activation blocks per stage
    constexpr int STAGE = (XB + kTN) * 1024;
    constexpr int PMIN = TM + 2;                      // copies per wave and k-step: TM + 2 (wave 0: + 3)
    static_assert(kNS * STAGE <= kParOff, "ring must not reach the epilogue operands");
    static_assert(2 * PMIN + 4 < 64, "vmcnt is a 6-bit counter");

    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int8_t *)smem;
#ifdef TRDQ_X_PROF
    const uint64_t prof_t0 = wall_clock64();
#endif
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lg = lane >> 4;
    const int KT = g.K >> 6;                          // k-steps
    const int64_t m0 = (int64_t)tm * BM;
    const int n0 = tn * kBN;

    const int64_t gstride = (int64_t)KT * 1024;      // bytes from one 16-row group to the next
    const int8_t *const xsrc = g.Xq + (m0 / 16 + wave * TM) * gstride;
    const int8_t *const wsrc = static_cast<const int8_t *>(g.Wc) + (int64_t)(n0 / 16) * gstride;
    const uint32_t voff = (uint32_t)blk_off(lane >> 2, lane & 3);

    const int8_t *xs[TM], *ws[2];
#pragma unroll
    for (int b = 0; b < TM; ++b) xs[b] = xsrc + b * gstride;
#pragma unroll
    for (int i = 0; i < 2; ++i) ws[i] = wsrc + (wave + 4 * i) * gstride;
    const int8_t *const ws8 = wsrc + 8 * gstride;     // the ninth weight block: wave 0 copies it
    // copy c (0 .. TM + 2) of this wave's share of k-step s into stage st: its TM activation blocks, two
    // weight blocks, and for wave 0 the ninth weight block
    auto issue_one = [&](auto c_tag, int s, int st) {
        constexpr int c = decltype(c_tag)::value;
        const uint32_t sbase = lds0 + st * STAGE;
        const int64_t so = (int64_t)s * 1024;
        if constexpr (c < TM) dma_1k(voff, xs[c] + so, sbase + (wave * TM + c) * 1024);
        else if constexpr (c < TM + 2) dma_1k(voff, ws[c - TM] + so, sbase + (XB + wave + 4 * (c - TM)) * 1024);
        else copy_1k_if(wave == 0, voff, ws8 + so, sbase + (XB + 8) * 1024);
    };
    auto issue = [&](int s, int st) {
        static_for_n<TM + 3>([&](auto c) { issue_one(c, s, st); });
    };

    // epilogue operands first (older than every tile copy, so the first wait covers them):
    // wave 0 the 144 channel scales, wave 1 the biases, wave 2 the BM token scales
    {
        const uint32_t par = lds0 + kParOff;
        const uint32_t v36 = (uint32_t)((lane < kBN / 4 ? lane : kBN / 4 - 1) * 16);
        const uint32_t vsx = (uint32_t)((lane < BM / 4 ? lane : BM / 4 - 1) * 16);
        copy_1k_if(wave == 0, v36, g.sw + n0, par + kParSw);
        copy_1k_if(wave == 1 && g.bias != nullptr, v36, g.bias ? g.bias + n0 : g.sw, par + kParBias);
        if (wave == 1 && g.bias == nullptr)           // no bias: zeros, so that the epilogue needs no branch
            *reinterpret_cast<uint4 *>(smem + kParOff + kParBias + lane * 16) = make_uint4(0u, 0u, 0u, 0u);
        copy_1k_if(wave == 2, vsx, g.sx + m0, par + kParSx);
    }
    // KT is even and at least 2 (K is a multiple of 128)
    issue(0, 0);
    issue(1, 1);
    if (KT >= 4) {
        issue(2, 2);
        wait_vmcnt<2 * PMIN>();
    } else {
        wait_vmcnt<PMIN>();
    }
    __syncthreads();

#ifdef TRDQ_X_PROF
    const uint64_t prof_t1 = wall_clock64();
#endif
    const int fro = blk_off(l16, lg);                 // the lane's piece of a fragment block
    v4i acc[kTN][TM];
#pragma unroll
    for (int a = 0; a < kTN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b) acc[a][b] = v4i{0, 0, 0, 0};
    v4i af[kTN], bf[2][TM];
#pragma unroll
    for (int a = 0; a < kTN; ++a) af[a] = *reinterpret_cast<const v4i *>(smem + (XB + a) * 1024 + fro);
#pragma unroll
    for (int b = 0; b < TM; ++b) bf[0][b] = *reinterpret_cast<const v4i *>(smem + (wave * TM + b) * 1024 + fro);

    int st = 0;
    // One k-step on activation fragment set PAR.  REFILL: the next step exists; its fragments are read
    // while this step's matrix instructions run (after waiting for vmcnt(WAITN) and the barrier).
    // ISSUE: the step three ahead exists and is requested into this step's stage.
    // The order below is the order of issue: the scheduling fences keep the compiler from bunching
    // the LDS reads at the end of the step, where nothing would cover their latency.
    auto step = [&](auto par_tag, auto refill_tag, auto issue_tag, auto wait_tag, int kt) {
        constexpr int PAR = decltype(par_tag)::value;
        constexpr bool REFILL = decltype(refill_tag)::value;
        constexpr bool ISSUE = decltype(issue_tag)::value;
        constexpr int WAITN = decltype(wait_tag)::value;
        const int nst = (st + 1 == kNS) ? 0 : st + 1;
        const int8_t *const nxt = smem + nst * STAGE + fro;
        if constexpr (REFILL) {
            wait_vmcnt<WAITN>();                               // step kt+1 has landed (this wave's share)
#ifndef TRDQ_X_NOBAR
            __syncthreads();                                   // ... everyone's; step kt's stage is retired
#endif
#ifndef TRDQ_X_NOCOPY
#endif
#pragma unroll
            for (int b = 0; b < TM; ++b)
                bf[1 - PAR][b] = *reinterpret_cast<const v4i *>(nxt + (wave * TM + b) * 1024);
            __builtin_amdgcn_sched_barrier(0);
        }
        static_for_n<kTN>([&](auto a_tag) {
            constexpr int a = decltype(a_tag)::value;
#pragma unroll
            for (int b = 0; b < TM; ++b)
#ifndef TRDQ_X_NOMFMA
                acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[a], bf[PAR][b], acc[a][b], 0, 0, 0);
#else
                acc[a][b] += af[a] ^ bf[PAR][b];
#endif
            if constexpr (REFILL) af[a] = *reinterpret_cast<const v4i *>(nxt + (XB + a) * 1024);
#ifndef TRDQ_X_NOCOPY
            // the copies of the step three ahead go out one at a time between the matrix instructions
            // (bunched, they stall the wave at the compute unit's copy path)
            if constexpr (ISSUE && a < TM + 3) issue_one(std::integral_constant<int, a>{}, kt + kNS, st);
#endif
            if constexpr (REFILL) __builtin_amdgcn_sched_barrier(0);
        });
        st = nst;
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using Yes = std::integral_constant<bool, true>;
    using No = std::integral_constant<bool, false>;
    using WP = std::integral_constant<int, PMIN>;
    if (KT >= 4) {
        int kt = 0;
        for (; kt + 4 < KT; kt += 2) {
            step(I0{}, Yes{}, Yes{}, WP{}, kt);
            step(I1{}, Yes{}, Yes{}, WP{}, kt + 1);
        }
        step(I0{}, Yes{}, Yes{}, WP{}, kt);           // kt = KT - 4: requests the last step
        step(I1{}, Yes{}, No{}, WP{}, kt + 1);
    }
    step(I0{}, Yes{}, No{}, I0{}, KT - 2);            // the last step's blocks: nothing younger is in flight
    step(I1{}, No{}, No{}, I0{}, KT - 1);

#ifdef TRDQ_X_PROF
    const uint64_t prof_t2 = wall_clock64();
#endif
    // ---- epilogue: y = float(acc) * s_x[m] * s_w[n] + bias[n] -> bf16.  One token tile (16 tokens x
    // 144 channels) at a time is laid out in the wave's part of the idle ring and read back row by
    // row, so that a store instruction writes whole 288-byte row segments, 16 bytes per lane.
    // (Laying out the wave's whole 64 x 144 block first and storing three rows per instruction cost
    // registers in the k-loop and was slower; the store phase is bound by the memory write rate.)
    __syncthreads();                                  // every wave has read its last fragments
    const float *const par = reinterpret_cast<const float *>(smem + kParOff);
    constexpr int ROWB = kBN * 2 + 16;
    int8_t *const stg = smem + wave * (16 * ROWB);
    const int64_t m_wave = m0 + wave * (BM / 4);
#pragma unroll
    for (int b = 0; b < TM; ++b) {
        const float sxm = par[kParSx / 4 + wave * (BM / 4) + b * 16 + l16];
#pragma unroll
        for (int a = 0; a < kTN; ++a) {
            const float4 s = *reinterpret_cast<const float4 *>(par + kParSw / 4 + a * 16 + lg * 4);
            const float4 bi = *reinterpret_cast<const float4 *>(par + kParBias / 4 + a * 16 + lg * 4);
            if constexpr (DEBUG) {
                const int64_t m = m_wave + b * 16 + l16;
                *reinterpret_cast<int4 *>(g.acc_debug + m * g.N + n0 + a * 16 + lg * 4) =
                    make_int4(acc[a][b][0], acc[a][b][1], acc[a][b][2], acc[a][b][3]);
            }
            uint2 o;
            o.x = pack_bf16x2((float)acc[a][b][0] * sxm * s.x + bi.x, (float)acc[a][b][1] * sxm * s.y + bi.y);
            o.y = pack_bf16x2((float)acc[a][b][2] * sxm * s.z + bi.z, (float)acc[a][b][3] * sxm * s.w + bi.w);
            *reinterpret_cast<uint2 *>(stg + l16 * ROWB + (a * 16 + lg * 4) * 2) = o;
        }
        __builtin_amdgcn_wave_barrier();
        constexpr int LPR = kBN / 8;
#pragma unroll
        for (int i = 0; i < (16 * LPR + 63) / 64; ++i) {
            const int id = i * 64 + lane;
            if (id < 16 * LPR) {
                const int row = id / LPR, c = id - row * LPR;
                const uint4 v = *reinterpret_cast<const uint4 *>(stg + row * ROWB + c * 16);
                store_out16(g.Y + (m_wave + b * 16 + row) * g.ldy + n0 + c * 8, v);
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
#ifdef TRDQ_X_PROF
    if (tid == 0 && g.acc_debug) {
        uint32_t hw, xcc;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
        uint64_t *o = reinterpret_cast<uint64_t *>(g.acc_debug) + (int64_t)blockIdx.x * 8;
        o[0] = prof_t0; o[1] = prof_t1; o[2] = prof_t2; o[3] = wall_clock64(); o[4] = hw; o[5] = xcc; o[6] = BM;
    }
#endif
}

template <bool DEBUG>
__global__ __launch_bounds__(kThreads, 2) void qgemm8_tiled_kernel(GemmArgs g, int n_big, int nbn)
{
    extern __shared__ __align__(16) int8_t smem[];
    const int id = blockIdx.x;
    const int tiles_n = g.N / kBN;
#ifdef TRDQ_X_PRIO
    if (id < (int)gridDim.x / 2) __builtin_amdgcn_s_setprio(3);
#endif
    int tm, tn;
    if (id < n_big) {
        tile_map(id, (int)(g.M / 256), nbn, tm, tn);
        run_tile<256, DEBUG>(g, tm, tn, smem);
    } else {
        tile_map(id - n_big, (int)(g.M / 128), tiles_n - nbn, tm, tn);
        run_tile<128, DEBUG>(g, tm, tn + nbn, smem);
    }
}

// 16 bytes per thread between the row-major form [R, K] and the block form
template <bool TO_TILED>
__global__ void retile_kernel(const int8_t *__restrict__ src, int8_t *__restrict__ dst, int64_t R, int K)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int cpr = K >> 4;                           // 16-byte pieces per row
    if (idx >= R * cpr) return;
    const int64_t row = idx / cpr;
    const int c = (int)(idx - row * cpr);
    const int64_t t = ((row >> 4) * (K >> 6) + (c >> 2)) * 1024 + (row & 15) * 64 + (c & 3) * 16;
    const int64_t r = row * K + (int64_t)c * 16;
    if (TO_TILED) *reinterpret_cast<uint4 *>(dst + t) = *reinterpret_cast<const uint4 *>(src + r);
    else *reinterpret_cast<uint4 *>(dst + r) = *reinterpret_cast<const uint4 *>(src + t);
}

}  // namespace

bool tiled_supports(const GemmArgs &a)
{
    return a.M > 0 && a.M % 128 == 0 && a.N % kBN == 0 && a.K % 128 == 0 && a.K >= 128 && a.ldy % 8 == 0 &&
           reinterpret_cast<uintptr_t>(a.Y) % 16 == 0 && !a.zc;
}

// How a launch splits the channel tiles between 256-token and 128-token workgroup tiles: the
// first nbn channel tiles go to tall tiles.  One round of two workgroups per compute unit if the
// short tiles alone would need more; all tall tiles when even those need more than one round.
void tiled_split(int64_t M, int N, int &n_big, int &nbn)
{
    const int T = N / kBN;
    const int64_t slots = 2 * (int64_t)num_cus();
    const int64_t p128 = M / 128;
    n_big = 0; nbn = 0;
#ifdef TRDQ_X_ALLSMALL
    return;
#endif
    if (M % 256 != 0 || p128 * T <= slots) return;
    // tiles(nbn) = (M / 256) * nbn + (M / 128) * (T - nbn) <= slots
    int64_t need = (p128 * T - slots + (p128 / 2) - 1) / (p128 / 2);
    nbn = (int)(need > T ? T : need);
    n_big = (int)((M / 256) * nbn);
}

hipError_t launch_qgemm8_tiled(const GemmArgs &a, bool debug, hipStream_t st)
{
    if (!tiled_supports(a)) return hipErrorInvalidValue;
    int n_big, nbn;
    tiled_split(a.M, a.N, n_big, nbn);
    const int64_t total = n_big + (a.M / 128) * (a.N / kBN - nbn);
    GemmArgs g = a;
    auto go = [&](auto kern) -> hipError_t {
        if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), kTiledLds); e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(kThreads), kTiledLds, st, g, n_big, nbn);
        return hipGetLastError();
    };
#ifdef TRDQ_X_PROF
    debug = false;                                    // the debug pointer receives time stamps instead
#endif
    return debug ? go(qgemm8_tiled_kernel<true>) : go(qgemm8_tiled_kernel<false>);
}

hipError_t launch_retile(const int8_t *src, int8_t *dst, int64_t R, int K, bool to_tiled, hipStream_t st)
{
    if (R <= 0) return hipSuccess;
    const int64_t n = R * (K / 16);
    const unsigned grid = (unsigned)((n + 255) / 256);
    if (to_tiled) hipLaunchKernelGGL(retile_kernel<true>, dim3(grid), dim3(256), 0, st, src, dst, R, K);
    else hipLaunchKernelGGL(retile_kernel<false>, dim3(grid), dim3(256), 0, st, src, dst, R, K);
    return hipGetLastError();
}

}  // namespace gemm
}  // namespace trdq
