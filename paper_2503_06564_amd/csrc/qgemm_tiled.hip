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
// of k (block (row / 16, k / 64) at ((row / 16) * K / 64 + k / 64) * 1024; inside a block the
// 16-byte piece p of row r at p * 256 + r * 16, the lane order of the matrix instruction's operand):
// one direct-to-LDS copy moves one block, eight whole cache lines, and one block is one operand
// fragment of v_mfma_i32_16x16x64_i8, read back from LDS as 1 KB in lane order.  trdq_rotate_quant_tiled writes activations in this form;
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
constexpr int kNS = 3;                       // stages of the ring
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

// A block in memory and in LDS: the 16-byte piece p (16 bytes of k) of row r sits at p * 256 + r * 16,
// which is lane (16 p + r)'s operand of the matrix instruction at 16 bytes per lane: a copy and a
// fragment read both move the block's 1 KB in lane order.
__device__ __forceinline__ int blk_off(int r, int p) { return p * 256 + r * 16; }

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
#ifdef TRDQ_PROBE_PHASES
    const uint64_t clk_c0 = __builtin_readcyclecounter();
    const uint64_t clk_t0 = wall_clock64();
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
    const uint32_t voff = (uint32_t)(lane * 16);        // copies keep the block's order

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

#ifdef TRDQ_PROBE_PHASES
    const uint64_t clk_c1 = __builtin_readcyclecounter();
    const uint64_t clk_t1 = wall_clock64();
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
            __syncthreads();                                   // ... everyone's; step kt's stage is retired
#pragma unroll
            for (int b = 0; b < TM; ++b)
                bf[1 - PAR][b] = *reinterpret_cast<const v4i *>(nxt + (wave * TM + b) * 1024);
            __builtin_amdgcn_sched_barrier(0);
        }
        static_for_n<kTN>([&](auto a_tag) {
            constexpr int a = decltype(a_tag)::value;
#pragma unroll
            for (int b = 0; b < TM; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[a], bf[PAR][b], acc[a][b], 0, 0, 0);
            if constexpr (REFILL) af[a] = *reinterpret_cast<const v4i *>(nxt + (XB + a) * 1024);
            // the copies of the step three ahead go out one at a time between the matrix instructions
            // (bunched, they stall the wave at the compute unit's copy path)
            if constexpr (ISSUE && a < TM + 3) issue_one(std::integral_constant<int, a>{}, kt + kNS, st);
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

#ifdef TRDQ_PROBE_PHASES
    const uint64_t clk_c2 = __builtin_readcyclecounter();
    const uint64_t clk_t2 = wall_clock64();
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
    // The lane's channel scales and biases are read one channel tile ahead of their use: read where
    // they are used, every one of the 9 x TM reads waits out an LDS round trip with nothing else to issue.
    const float *const psw = par + kParSw / 4 + lg * 4, *const pbi = par + kParBias / 4 + lg * 4;
    float4 s_nxt = *reinterpret_cast<const float4 *>(psw), bi_nxt = *reinterpret_cast<const float4 *>(pbi);
#pragma unroll
    for (int b = 0; b < TM; ++b) {
        const float sxm = par[kParSx / 4 + wave * (BM / 4) + b * 16 + l16];
#pragma unroll
        for (int a = 0; a < kTN; ++a) {
            const float4 s = s_nxt, bi = bi_nxt;
            {
                const int an = (a + 1) % kTN;         // wraps to the first tile for the next token tile
                s_nxt = *reinterpret_cast<const float4 *>(psw + an * 16);
                bi_nxt = *reinterpret_cast<const float4 *>(pbi + an * 16);
            }
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
#ifdef TRDQ_PROBE_PHASES
    if (tid == 0 && g.acc_debug) {
        const uint64_t clk_c3 = __builtin_readcyclecounter();
        uint32_t hw, xcc;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
        uint64_t *o = reinterpret_cast<uint64_t *>(g.acc_debug) + (int64_t)blockIdx.x * 16;
        o[0] = clk_t0; o[1] = clk_t1; o[2] = clk_t2; o[3] = wall_clock64();
        o[4] = clk_c0; o[5] = clk_c1; o[6] = clk_c2; o[7] = clk_c3;
        o[8] = hw; o[9] = xcc; o[10] = BM; o[11] = 1;
    }
#endif
}

template <bool DEBUG>
__global__ __launch_bounds__(kThreads, 2) void qgemm8_tiled_kernel(GemmArgs g, int n_big, int nbn)
{
    extern __shared__ __align__(16) int8_t smem[];
    const int id = blockIdx.x;
    const int tiles_n = g.N / kBN;
    int tm, tn;
    if (id < n_big) {
        tile_map(id, (int)(g.M / 256), nbn, tm, tn);
        run_tile<256, DEBUG>(g, tm, tn, smem);
    } else {
        tile_map(id - n_big, (int)(g.M / 128), tiles_n - nbn, tm, tn);
        run_tile<128, DEBUG>(g, tm, tn + nbn, smem);
    }
}

// ---- one tile per compute unit: K split over two wave pairs --------------------------------------
// A launch with no more 128 x 144 tiles than compute units has nothing to put beside a tile, and a
// 128-token tile run by four waves as above means wave tiles of 32 x 144, whose fragment reads
// (0.6 KB per matrix instruction) bound the loop.  Here the four waves share the tile as two token
// halves x two halves of K: every wave keeps the 64 x 144 wave tile, each pair walks its half of
// the k-steps on a ring of its own (NS stages of 17 KB: 8 activation + 9 weight blocks), and all
// four meet at one barrier per k-step.  Such a tile pulls 17 KB through the compute unit's copy
// path per 72 matrix instructions, and that path delivers about 120 KB/us with nothing else going
// on (measured), so the loop runs at the rate of the copies and what counts is how many of them
// are in flight: two pairs x four stages keep three quarters of a 136 KB ring in flight (four
// pairs x two stages, eight waves, kept half of it and was 20 % slower; whether the blocks came
// from L2 or from behind it made no difference).
// At the end the two partial sums of each token sub-tile (16 tokens x 144 channels) meet in LDS,
// each pair adding up and finishing two of the four sub-tiles of both token halves.
// Needs K % 128 == 0 (the same number of k-steps for both pairs) and at least NS k-steps per pair;
// NS is 4, or 3 where the number of k-steps per pair is odd (the main loop takes two at a time).
constexpr int kKsStage = (8 + kTN) * 1024;
constexpr int kKsCopies = 9;                         // per wave and k-step
constexpr int kKsPairs = 2;
template <int NS> constexpr int ks_par_off() { return kKsPairs * NS * kKsStage; }
template <int NS> constexpr int ks_lds() { return ks_par_off<NS>() + 3072; }

template <int NS, bool DEBUG>
__global__ __launch_bounds__(128 * kKsPairs) void qgemm8_tiled_ksplit_kernel(GemmArgs g)
{
    constexpr int NG = kKsPairs;
    extern __shared__ __align__(16) int8_t smem[];
    constexpr int TM = 4;
    constexpr int P = kKsCopies;
    constexpr int RING = NS * kKsStage;
    constexpr int PAROFF = ks_par_off<NS>();
    static_assert((NS - 1) * P < 64, "vmcnt is a 6-bit counter");
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int8_t *)smem;
#ifdef TRDQ_PROBE_PHASES
    const uint64_t clk_c0 = __builtin_readcyclecounter();
    const uint64_t clk_t0 = wall_clock64();
#endif
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int mw = wave & 1, kg = wave >> 1;         // token half, part of K
    const int l16 = lane & 15, lg = lane >> 4;
    int tm, tn;
    tile_map(blockIdx.x, (int)(g.M / 128), g.N / kBN, tm, tn);
    const int KT = g.K >> 6;                          // k-steps of the product
    const int KTg = KT / NG;                          // of one pair: even, at least NS
    const int64_t m0 = (int64_t)tm * 128;
    const int n0 = tn * kBN;

    const int64_t gstride = (int64_t)KT * 1024;      // bytes from one 16-row group to the next
    const int64_t kofs = (int64_t)kg * KTg * 1024;   // this pair's first k-step
    const int8_t *const xsrc = g.Xq + (m0 / 16 + mw * TM) * gstride + kofs;
    const int8_t *const wsrc = static_cast<const int8_t *>(g.Wc) + (int64_t)(n0 / 16) * gstride + kofs;
    const uint32_t voff = (uint32_t)(lane * 16);        // copies keep the block's order
    int8_t *const ring = smem + kg * RING;
    const uint32_t ring0 = lds0 + kg * RING;

    // this wave's nine copies of a k-step: its own four activation blocks, and weight blocks 0..4
    // (first wave of the pair) or 5..8 and 8 once more (second wave: equal counts keep the waits uniform)
    const int8_t *src[P];
    uint32_t dst[P];
#pragma unroll
    for (int b = 0; b < TM; ++b) {
        src[b] = xsrc + b * gstride;
        dst[b] = (uint32_t)((mw * TM + b) * 1024);
    }
#pragma unroll
    for (int i = 0; i < P - TM; ++i) {
        const int blk = mw == 0 ? i : (5 + i < kTN ? 5 + i : kTN - 1);
        src[TM + i] = wsrc + blk * gstride;
        dst[TM + i] = (uint32_t)((8 + blk) * 1024);
    }
    auto issue_one = [&](auto c_tag, int s, int st) {
        constexpr int c = decltype(c_tag)::value;
        dma_1k(voff, src[c] + (int64_t)s * 1024, ring0 + st * kKsStage + dst[c]);
    };
    auto issue = [&](int s, int st) {
        static_for_n<P>([&](auto c) { issue_one(c, s, st); });
    };

    // epilogue operands first (older than every tile copy, so the first wait covers them)
    {
        const uint32_t par = lds0 + PAROFF;
        const uint32_t v36 = (uint32_t)((lane < kBN / 4 ? lane : kBN / 4 - 1) * 16);
        const uint32_t vsx = (uint32_t)((lane < 128 / 4 ? lane : 128 / 4 - 1) * 16);
        copy_1k_if(wave == 0, v36, g.sw + n0, par + kParSw);
        copy_1k_if(wave == 1 && g.bias != nullptr, v36, g.bias ? g.bias + n0 : g.sw, par + kParBias);
        if (wave == 1 && g.bias == nullptr)
            *reinterpret_cast<uint4 *>(smem + PAROFF + kParBias + lane * 16) = make_uint4(0u, 0u, 0u, 0u);
        copy_1k_if(wave == 2, vsx, g.sx + m0, par + kParSx);
    }
#pragma unroll
    for (int s = 0; s < NS; ++s) issue(s, s);
    wait_vmcnt<(NS - 1) * P>();                       // step 0 and the operands above
    __syncthreads();
#ifdef TRDQ_PROBE_PHASES
    const uint64_t clk_c1 = __builtin_readcyclecounter();
    const uint64_t clk_t1 = wall_clock64();
#endif

    const int fro = blk_off(l16, lg);
    v4i acc[kTN][TM];
#pragma unroll
    for (int a = 0; a < kTN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b) acc[a][b] = v4i{0, 0, 0, 0};
    v4i af[kTN], bf[2][TM];
#pragma unroll
    for (int a = 0; a < kTN; ++a) af[a] = *reinterpret_cast<const v4i *>(ring + (8 + a) * 1024 + fro);
#pragma unroll
    for (int b = 0; b < TM; ++b) bf[0][b] = *reinterpret_cast<const v4i *>(ring + (mw * TM + b) * 1024 + fro);

    int st = 0;
    // One k-step on activation fragment set PAR.  REFILL: the next step exists: wait until at most
    // WAITN younger copies are in flight (then it has landed), barrier, and read its fragments while
    // this step's matrix instructions run.  ISSUE: the step NS ahead exists and is requested into
    // this step's stage, whose fragments are all in registers by now.
    auto step = [&](auto par_tag, auto refill_tag, auto issue_tag, auto wait_tag, int kt) {
        constexpr int PAR = decltype(par_tag)::value;
        constexpr bool REFILL = decltype(refill_tag)::value;
        constexpr bool ISSUE = decltype(issue_tag)::value;
        constexpr int WAITN = decltype(wait_tag)::value;
        const int nst = (st + 1 == NS) ? 0 : st + 1;
        const int8_t *const nxt = ring + nst * kKsStage + fro;
        if constexpr (REFILL) {
            wait_vmcnt<WAITN>();
            __syncthreads();
#pragma unroll
            for (int b = 0; b < TM; ++b)
                bf[1 - PAR][b] = *reinterpret_cast<const v4i *>(nxt + (mw * TM + b) * 1024);
            __builtin_amdgcn_sched_barrier(0);
        }
        static_for_n<kTN>([&](auto a_tag) {
            constexpr int a = decltype(a_tag)::value;
#pragma unroll
            for (int b = 0; b < TM; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[a], bf[PAR][b], acc[a][b], 0, 0, 0);
            if constexpr (REFILL) af[a] = *reinterpret_cast<const v4i *>(nxt + (8 + a) * 1024);
            if constexpr (ISSUE && a < P) issue_one(std::integral_constant<int, a>{}, kt + NS, st);
            if constexpr (REFILL) __builtin_amdgcn_sched_barrier(0);
        });
        st = nst;
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using Yes = std::integral_constant<bool, true>;
    using No = std::integral_constant<bool, false>;
    using WFull = std::integral_constant<int, (NS - 2) * P>;
    int kt = 0;
    for (; kt + NS < KTg; kt += 2) {                  // KTg - NS is even (the launcher picks NS by the parity of KTg)
        step(I0{}, Yes{}, Yes{}, WFull{}, kt);
        step(I1{}, Yes{}, Yes{}, WFull{}, kt + 1);
    }
    // the last NS steps request nothing; step j of them leaves NS - 2 - j younger steps in flight
    static_for_n<NS>([&](auto j_tag) {
        constexpr int j = decltype(j_tag)::value;
        using Par = std::integral_constant<int, j & 1>;
        if constexpr (j + 1 < NS) step(Par{}, Yes{}, No{}, std::integral_constant<int, (NS - 2 - j) * P>{}, kt + j);
        else step(Par{}, No{}, No{}, I0{}, kt + j);
    });

#ifdef TRDQ_PROBE_PHASES
    const uint64_t clk_c2 = __builtin_readcyclecounter();
    const uint64_t clk_t2 = wall_clock64();
#endif
    // ---- the partial sums of every token sub-tile meet in LDS ------------------------------------
    __syncthreads();                                  // every wave has read its last fragments
    v4i *const xch = reinterpret_cast<v4i *>(smem);
    constexpr int ROWB = kBN * 2 + 16;
    int8_t *stg;
    {
        // Pair q finishes sub-tiles 2q, 2q + 1: each wave lays down the two it does not finish
        // ([4 waves][2][9][64]) and adds what the other pair's wave of its token half left for it.
        {
            v4i *const out = xch + (wave * 2 * kTN) * 64 + lane;
#pragma unroll
            for (int a = 0; a < kTN; ++a) {
                out[a * 64] = kg == 0 ? acc[a][2] : acc[a][0];
                out[(kTN + a) * 64] = kg == 0 ? acc[a][3] : acc[a][1];
            }
        }
        __syncthreads();
        {
            const v4i *const in = xch + (((1 - kg) * 2 + mw) * 2 * kTN) * 64 + lane;
#pragma unroll
            for (int a = 0; a < kTN; ++a) {
                const v4i p0 = in[a * 64], p1 = in[(kTN + a) * 64];
                if (kg == 0) { acc[a][0] += p0; acc[a][1] += p1; }
                else { acc[a][2] += p0; acc[a][3] += p1; }
            }
        }
        stg = smem + 4 * 2 * kTN * 1024 + wave * (16 * ROWB);   // behind the exchange area
    }

    // ---- epilogue of this wave's sub-tiles: 16 tokens x all 144 channels each ---------------------
    const float *const par = reinterpret_cast<const float *>(smem + PAROFF);
    float4 sw_r[kTN], bi_r[kTN];                      // the lane's channel scales and biases, read once
#pragma unroll
    for (int a = 0; a < kTN; ++a) {
        sw_r[a] = *reinterpret_cast<const float4 *>(par + kParSw / 4 + a * 16 + lg * 4);
        bi_r[a] = *reinterpret_cast<const float4 *>(par + kParBias / 4 + a * 16 + lg * 4);
    }
    static_for_n<TM>([&](auto b_tag) {
        constexpr int b = decltype(b_tag)::value;
        if (b * NG / TM == kg) {                      // wave-uniform
            const int64_t m_own = m0 + mw * 64 + b * 16;
            const float sxm = par[kParSx / 4 + mw * 64 + b * 16 + l16];
#pragma unroll
            for (int a = 0; a < kTN; ++a) {
                const float4 s = sw_r[a];
                const float4 bi = bi_r[a];
                if constexpr (DEBUG) {
                    *reinterpret_cast<int4 *>(g.acc_debug + (m_own + l16) * g.N + n0 + a * 16 + lg * 4) =
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
                    store_out16(g.Y + (m_own + row) * g.ldy + n0 + c * 8, v);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    });
#ifdef TRDQ_PROBE_PHASES
    if (tid == 0 && g.acc_debug) {
        const uint64_t clk_c3 = __builtin_readcyclecounter();
        uint32_t hw, xcc;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
        uint64_t *o = reinterpret_cast<uint64_t *>(g.acc_debug) + (int64_t)blockIdx.x * 16;
        o[0] = clk_t0; o[1] = clk_t1; o[2] = clk_t2; o[3] = wall_clock64();
        o[4] = clk_c0; o[5] = clk_c1; o[6] = clk_c2; o[7] = clk_c3;
        o[8] = hw; o[9] = xcc; o[10] = 128; o[11] = 2;                 // 2: the K-split kernel
    }
#endif
}

// ---- int4 weights on block-tiled operands ---------------------------------------------------------
// Eq. 10's product with 4-bit weight codes and one scale per 128 input channels and output channel.
// Activations as above (1 KB blocks).  Weights: the 8 packed bytes that hold 16 consecutive input
// channels of one output channel (byte j of a 4-byte word = code(k0 + j) | code(k0 + 4 + j) << 4, as
// in the row-major form) are the unit; a block is 16 output channels x 64 input channels = 512 bytes,
// unit (n, q = k / 16) at ((n / 16) * (K / 64) + q / 4) * 512 + (q % 4) * 128 + (n % 16) * 8: lane order
// again, 8 bytes per lane.  A lane widens its unit to 16 * code in registers (one shift-and-mask and
// one mask per word), the matrix instruction is the int8 one, and after the two k-steps of a scale
// group the int32 sums are folded into float accumulators with the group's scales; the factor 16
// leaves with the token scale in the epilogue.
//
// 128 x 128 tiles, four waves as 2 x 2 (64 x 64 wave tiles: 64 + 64 accumulator registers), two
// workgroups per compute unit, a ring of five stages of 13 KB (8 activation blocks, 8 weight blocks, the
// group's 128 scales).  Per wave and k-step four copies: two activation blocks, 1 KB of weight blocks
// (two of them), 256 bytes of scales (waves 2 and 3 copy them a second time into a spare area, and
// the scales travel with both k-steps of their group, so that every wave issues the same number of
// requests per step; past the last k-step the last one is copied again, for the same reason).
// The fold of group g is spread over the first k-step of group g + 1: tile by tile, the eight vector
// instructions of a tile right before the matrix instruction that starts the tile's next sum from
// zero, so that they run under the matrix instructions of the tiles before.
constexpr int kW4BM = 128, kW4BN = 128;
constexpr int kW4NS = 5;
constexpr int kW4XOff = 0, kW4WOff = 8192, kW4SOff = 12288;
constexpr int kW4Stage = 13312;
constexpr int kW4ParOff = kW4NS * kW4Stage;          // epilogue operands: [128 bias][128 s_x]
constexpr int kW4Lds = kW4ParOff + 2048;             // 68608 B
constexpr int kW4Copies = 4;

__device__ __forceinline__ void copy_256_if(int on, uint32_t voff, const void *sbase, uint32_t lds_addr)
{
    asm volatile("s_cmp_eq_u32 %3, 0\n\ts_cbranch_scc1 .Lskip%=\n\t"
                 "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1\n"
                 ".Lskip%=:"
                 :: "v"(voff), "s"(sbase), "s"(lds_addr), "s"(__builtin_amdgcn_readfirstlane(on))
                 : "memory", "scc");
}

template <bool DEBUG>
__global__ __launch_bounds__(kThreads, 2) void qgemm4_tiled_kernel(GemmArgs g)
{
    extern __shared__ __align__(16) int8_t smem[];
    constexpr int TM = 4, TN = 4, NS = kW4NS, P = kW4Copies;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int8_t *)smem;
#ifdef TRDQ_PROBE_PHASES
    const uint64_t clk_c0 = __builtin_readcyclecounter();
    const uint64_t clk_t0 = wall_clock64();
#endif
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int l16 = lane & 15, lg = lane >> 4;
    int tm, tn;
    tile_map(blockIdx.x, (int)(g.M / kW4BM), g.N / kW4BN, tm, tn);
    const int KT = g.K >> 6;                          // k-steps: even, at least NS
    const int64_t m0 = (int64_t)tm * kW4BM;
    const int n0 = tn * kW4BN;

    const int64_t xstride = (int64_t)KT * 1024;      // bytes from one 16-token group to the next
    const int64_t wstride = (int64_t)KT * 512;       // ... one 16-channel group to the next
    const int8_t *const xsrc = g.Xq + (m0 / 16 + 2 * wave) * xstride;
    const uint8_t *const wsrc = static_cast<const uint8_t *>(g.Wc) + (int64_t)(n0 / 16 + 2 * wave) * wstride;
    const uint32_t voff = (uint32_t)(lane * 16);
    // the weight copy moves two blocks: lanes 0-31 the first, lanes 32-63 the one a channel group further
    const uint32_t voffw = (uint32_t)((lane & 31) * 16) + (lane >= 32 ? (uint32_t)wstride : 0u);
    const float *const ssrc = g.sw + n0 + (wave & 1) * 64;
    const uint32_t voffs = (uint32_t)(lane * 4);
    auto issue_one = [&](auto c_tag, int s, int st) {
        constexpr int c = decltype(c_tag)::value;
        const uint32_t sbase = lds0 + st * kW4Stage;
        if constexpr (c < 2) dma_1k(voff, xsrc + c * xstride + (int64_t)s * 1024, sbase + kW4XOff + (2 * wave + c) * 1024);
        else if constexpr (c == 2) dma_1k(voffw, wsrc + (int64_t)s * 512, sbase + kW4WOff + wave * 1024);
        else copy_256_if(1, voffs, ssrc + (int64_t)(s >> 1) * g.N, sbase + kW4SOff + wave * 256);
    };
    auto issue = [&](int s, int st) {
        static_for_n<P>([&](auto c) { issue_one(c, s, st); });
    };

    // epilogue operands first: wave 0 the biases, wave 1 the token scales (half a copy each)
    {
        const uint32_t par = lds0 + kW4ParOff;
        const uint32_t v32 = (uint32_t)((lane & 31) * 16);
        copy_1k_if(wave == 0 && g.bias != nullptr, v32, g.bias ? g.bias + n0 : g.sw, par);
        if (wave == 0 && g.bias == nullptr)
            *reinterpret_cast<uint4 *>(smem + kW4ParOff + lane * 16) = make_uint4(0u, 0u, 0u, 0u);
        copy_1k_if(wave == 1, v32, g.sx + m0, par + 1024);
    }
#pragma unroll
    for (int s = 0; s < NS; ++s) issue(s, s);
    wait_vmcnt<(NS - 1) * P>();
    __syncthreads();
#ifdef TRDQ_PROBE_PHASES
    const uint64_t clk_c1 = __builtin_readcyclecounter();
    const uint64_t clk_t1 = wall_clock64();
#endif

    const int xfr = kW4XOff + (wm * TM) * 1024 + lane * 16;
    const int wfr = kW4WOff + (wn * TN) * 512 + lane * 8;
    const int sfr = kW4SOff + (wn * 64 + lg * 4) * 4;
    auto widen = [](uint2 p) {
        return v4i{(int)((p.x << 4) & 0xF0F0F0F0u), (int)(p.x & 0xF0F0F0F0u),
                   (int)((p.y << 4) & 0xF0F0F0F0u), (int)(p.y & 0xF0F0F0F0u)};
    };
    v4i acc[TN][TM];
    v4f facc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b) { acc[a][b] = v4i{0, 0, 0, 0}; facc[a][b] = v4f{0.f, 0.f, 0.f, 0.f}; }
    v4i af[TN], bf[2][TM];
    uint2 raw[TN];
    float4 sc[TN];
#pragma unroll
    for (int a = 0; a < TN; ++a) {
        af[a] = widen(*reinterpret_cast<const uint2 *>(smem + wfr + a * 512));
        sc[a] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int b = 0; b < TM; ++b) bf[0][b] = *reinterpret_cast<const v4i *>(smem + xfr + b * 1024);

    const int n_lane = n0 + wn * 64 + lg * 4;
    const int64_t m_lane0 = m0 + wm * 64 + l16;
    int st = 0;
    // One k-step.  HALF 0 starts the sums of a scale group (folding the group before, tile by tile, with
    // the scales read one group earlier) and ends by reading the new group's scales; HALF 1 continues the sums.
    auto step = [&](auto half_tag, auto fold_tag, auto next_tag, int kt) {
        constexpr int HALF = decltype(half_tag)::value;
        constexpr bool fold_prev = decltype(fold_tag)::value;     // a group before this one exists
        constexpr bool has_next = decltype(next_tag)::value;      // a k-step after this one exists
        const int nst = (st + 1 == NS) ? 0 : st + 1;
        const int8_t *const nxt = smem + nst * kW4Stage;
        wait_vmcnt<(NS - 2) * P>();
        __syncthreads();
        if constexpr (has_next) {
#pragma unroll
            for (int b = 0; b < TM; ++b) bf[1 - HALF][b] = *reinterpret_cast<const v4i *>(nxt + xfr + b * 1024);
#pragma unroll
            for (int a = 0; a < TN; ++a) raw[a] = *reinterpret_cast<const uint2 *>(nxt + wfr + a * 512);
        }
        __builtin_amdgcn_sched_barrier(0);
        static_for_n<TN>([&](auto a_tag) {
            constexpr int a = decltype(a_tag)::value;
#pragma unroll
            for (int b = 0; b < TM; ++b) {
                if constexpr (HALF == 0) {
                    if constexpr (fold_prev) {
                        if constexpr (DEBUG) {
                            const int64_t m = m_lane0 + b * 16;
                            *reinterpret_cast<int4 *>(g.acc_debug + ((int64_t)((kt >> 1) - 1) * g.M + m) * g.N + n_lane + a * 16) =
                                make_int4(acc[a][b][0] >> 4, acc[a][b][1] >> 4, acc[a][b][2] >> 4, acc[a][b][3] >> 4);
                        }
                        facc[a][b][0] += sc[a].x * (float)acc[a][b][0];
                        facc[a][b][1] += sc[a].y * (float)acc[a][b][1];
                        facc[a][b][2] += sc[a].z * (float)acc[a][b][2];
                        facc[a][b][3] += sc[a].w * (float)acc[a][b][3];
                    }
                    acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[a], bf[HALF][b], v4i{0, 0, 0, 0}, 0, 0, 0);
                } else {
                    acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[a], bf[HALF][b], acc[a][b], 0, 0, 0);
                }
            }
            if constexpr (has_next) af[a] = widen(raw[a]);
            issue_one(std::integral_constant<int, a>{}, kt + NS < KT ? kt + NS : KT - 1, st);
            __builtin_amdgcn_sched_barrier(0);
        });
        // The group's scales, once the fold of the group before is done, from the NEXT step's stage (they
        // travel with both steps of the group): that stage is not given away before the next barrier,
        // this step's is being refilled by the other waves already.
        if constexpr (HALF == 0) {
#pragma unroll
            for (int a = 0; a < TN; ++a) sc[a] = *reinterpret_cast<const float4 *>(nxt + sfr + a * 64);
        }
        st = nst;
    };
    using H0 = std::integral_constant<int, 0>;
    using H1 = std::integral_constant<int, 1>;
    using Yes = std::integral_constant<bool, true>;
    using No = std::integral_constant<bool, false>;
    step(H0{}, No{}, Yes{}, 0);                       // at least three groups (the launcher checks)
    step(H1{}, No{}, Yes{}, 1);
    int kt = 2;
    for (; kt + 2 < KT; kt += 2) {
        step(H0{}, Yes{}, Yes{}, kt);
        step(H1{}, No{}, Yes{}, kt + 1);
    }
    step(H0{}, Yes{}, Yes{}, kt);
    step(H1{}, No{}, No{}, kt + 1);
    wait_vmcnt<0>();                                  // the repeated copies of the last steps
#ifdef TRDQ_PROBE_PHASES
    const uint64_t clk_c2 = __builtin_readcyclecounter();
    const uint64_t clk_t2 = wall_clock64();
#endif
    // the last group's fold
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b) {
            if constexpr (DEBUG) {
                const int64_t m = m_lane0 + b * 16;
                *reinterpret_cast<int4 *>(g.acc_debug + ((int64_t)((KT >> 1) - 1) * g.M + m) * g.N + n_lane + a * 16) =
                    make_int4(acc[a][b][0] >> 4, acc[a][b][1] >> 4, acc[a][b][2] >> 4, acc[a][b][3] >> 4);
            }
            facc[a][b][0] += sc[a].x * (float)acc[a][b][0];
            facc[a][b][1] += sc[a].y * (float)acc[a][b][1];
            facc[a][b][2] += sc[a].z * (float)acc[a][b][2];
            facc[a][b][3] += sc[a].w * (float)acc[a][b][3];
        }

    // ---- epilogue: y = (s_x / 16) * facc + bias -> bf16, one 16-token tile at a time through the idle ring
    __syncthreads();
    const float *const par = reinterpret_cast<const float *>(smem + kW4ParOff);
    constexpr int ROWB = 64 * 2 + 16;                 // a wave's 64 channels of one token, padded
    int8_t *const stg = smem + wave * (16 * ROWB);
    float4 bi_r[TN];
#pragma unroll
    for (int a = 0; a < TN; ++a) bi_r[a] = *reinterpret_cast<const float4 *>(par + wn * 64 + a * 16 + lg * 4);
#pragma unroll
    for (int b = 0; b < TM; ++b) {
        const float sxm = par[256 + wm * 64 + b * 16 + l16] * 0.0625f;
#pragma unroll
        for (int a = 0; a < TN; ++a) {
            uint2 o;
            o.x = pack_bf16x2(sxm * facc[a][b][0] + bi_r[a].x, sxm * facc[a][b][1] + bi_r[a].y);
            o.y = pack_bf16x2(sxm * facc[a][b][2] + bi_r[a].z, sxm * facc[a][b][3] + bi_r[a].w);
            *reinterpret_cast<uint2 *>(stg + l16 * ROWB + (a * 16 + lg * 4) * 2) = o;
        }
        __builtin_amdgcn_wave_barrier();
        // 16 rows x 128 bytes = 128 pieces of 16 bytes: two per lane
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int id = i * 64 + lane;
            const int row = id >> 3, c = id & 7;
            const uint4 v = *reinterpret_cast<const uint4 *>(stg + row * ROWB + c * 16);
            store_out16(g.Y + (m0 + wm * 64 + b * 16 + row) * g.ldy + n0 + wn * 64 + c * 8, v);
        }
        __builtin_amdgcn_wave_barrier();
    }
#ifdef TRDQ_PROBE_PHASES
    if (tid == 0 && g.acc_debug) {
        const uint64_t clk_c3 = __builtin_readcyclecounter();
        uint32_t hw, xcc;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
        uint64_t *o = reinterpret_cast<uint64_t *>(g.acc_debug) + (int64_t)blockIdx.x * 16;
        o[0] = clk_t0; o[1] = clk_t1; o[2] = clk_t2; o[3] = wall_clock64();
        o[4] = clk_c0; o[5] = clk_c1; o[6] = clk_c2; o[7] = clk_c3;
        o[8] = hw; o[9] = xcc; o[10] = 128; o[11] = 4;                 // 4: the int4 kernel
    }
#endif
}

// 8-byte units between the row-major packed form [N, K / 2] and the block form above
__global__ void retile_w4_kernel(const uint2 *__restrict__ src, uint2 *__restrict__ dst, int64_t N, int K)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int upr = K >> 4;                           // units per channel
    if (idx >= N * upr) return;
    const int64_t n = idx / upr;
    const int q = (int)(idx - n * upr);
    const int64_t t = ((n >> 4) * (K >> 6) + (q >> 2)) * 64 + (q & 3) * 16 + (n & 15);
    dst[t] = src[idx];
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
    const int64_t t = ((row >> 4) * (K >> 6) + (c >> 2)) * 1024 + (c & 3) * 256 + (row & 15) * 16;
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
    if (M % 256 != 0 || p128 * T <= slots) return;
    // tiles(nbn) = (M / 256) * nbn + (M / 128) * (T - nbn) <= slots
    int64_t need = (p128 * T - slots + (p128 / 2) - 1) / (p128 / 2);
    nbn = (int)(need > T ? T : need);
    n_big = (int)((M / 256) * nbn);
}

// The kernel that splits K inside the workgroup: two pairs, four stages for an even number of
// k-steps per pair and three for an odd one (the main loop takes the steps two at a time).
bool tiled_ksplit_applies(const GemmArgs &a)
{
    return a.K % 128 == 0 && a.K >= 1024 && (a.M / 128) * (int64_t)(a.N / kBN) <= num_cus();
}

template <int NS>
hipError_t launch_ksplit(const GemmArgs &a, bool debug, hipStream_t st)
{
    GemmArgs g = a;
    constexpr int lds = ks_lds<NS>();
    auto go = [&](auto kern) -> hipError_t {
        if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), lds); e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3((unsigned)((a.M / 128) * (a.N / kBN))), dim3(256), lds, st, g);
        return hipGetLastError();
    };
#ifdef TRDQ_PROBE_PHASES
    debug = false;                                    // the debug pointer receives time stamps instead
#endif
    return debug ? go(qgemm8_tiled_ksplit_kernel<NS, true>) : go(qgemm8_tiled_ksplit_kernel<NS, false>);
}

hipError_t launch_qgemm8_tiled(const GemmArgs &a, bool debug, hipStream_t st)
{
    if (!tiled_supports(a)) return hipErrorInvalidValue;
    if (tiled_ksplit_applies(a)) return ((a.K / 128) & 1) ? launch_ksplit<3>(a, debug, st) : launch_ksplit<4>(a, debug, st);
    int n_big, nbn;
    tiled_split(a.M, a.N, n_big, nbn);
    const int64_t total = n_big + (a.M / 128) * (a.N / kBN - nbn);
    GemmArgs g = a;
    auto go = [&](auto kern) -> hipError_t {
        if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), kTiledLds); e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(kThreads), kTiledLds, st, g, n_big, nbn);
        return hipGetLastError();
    };
#ifdef TRDQ_PROBE_PHASES
    debug = false;                                    // the debug pointer receives time stamps instead
#endif
    return debug ? go(qgemm8_tiled_kernel<true>) : go(qgemm8_tiled_kernel<false>);
}

bool tiled4_supports(const GemmArgs &a)
{
    return a.M > 0 && a.M % kW4BM == 0 && a.N % kW4BN == 0 && a.K % 128 == 0 && a.K >= 64 * kW4NS + 64 && a.ldy % 8 == 0 &&
           reinterpret_cast<uintptr_t>(a.Y) % 16 == 0 && !a.zc;
}

hipError_t launch_qgemm4_tiled(const GemmArgs &a, bool debug, hipStream_t st)
{
    if (!tiled4_supports(a)) return hipErrorInvalidValue;
    GemmArgs g = a;
    auto go = [&](auto kern) -> hipError_t {
        if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), kW4Lds); e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3((unsigned)((a.M / kW4BM) * (a.N / kW4BN))), dim3(kThreads), kW4Lds, st, g);
        return hipGetLastError();
    };
#ifdef TRDQ_PROBE_PHASES
    debug = false;                                    // the debug pointer receives time stamps instead
#endif
    return debug ? go(qgemm4_tiled_kernel<true>) : go(qgemm4_tiled_kernel<false>);
}

hipError_t launch_retile_w4(const void *src, void *dst, int64_t N, int K, hipStream_t st)
{
    const int64_t n = N * (K / 16);
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(retile_w4_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                       static_cast<const uint2 *>(src), static_cast<uint2 *>(dst), N, K);
    return hipGetLastError();
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
