// W8A8 integer product with a 256 x 256 output tile per workgroup and a hand-scheduled main loop.
//
// Why this shape: with int8 matrix instructions at 2048 ops per clock per SIMD the kernel is
// bound by what the L2 can deliver to the compute units, so the tile is the largest one the
// register file allows (four waves, each 128 channels x 128 tokens = 256 accumulator registers),
// which halves the operand bytes per operation of a 128 x 128 tile.  One wave per SIMD means
// nothing else hides instruction-issue bubbles, so the k-loop is written in assembly: 64 matrix
// instructions per 64-deep k-step with the 16 LDS fragment reads of the next step and the 8
// direct-to-LDS copies of a later k-step placed between them at fixed intervals, accumulators in
// the accumulation registers a0-a255, fragments double-buffered in v128-v255.
//
// Operation: Y = dequant(Xq . Wq^T) of Eq. 10's quantised product, per-token and per-channel
// scales, optional bias, bf16 output (the same arithmetic as the other int8 kernels).
#include "gemm_common.h"

#include <type_traits>
#include <utility>

namespace trdq {
namespace gemm {

namespace {

constexpr int kWideBM = 256;                 // tokens per tile
constexpr int kWideBN = 256;                 // output channels per tile
constexpr int kWideBK = 64;                  // bytes of k per k-step (one matrix instruction deep)
constexpr int kWideSlot = (kWideBM + kWideBN) * kWideBK;    // 32 KB: [tokens 256 x 64][channels 256 x 64]
constexpr int kWideSlots = 5;
constexpr int kWideLds = kWideSlots * kWideSlot;            // 160 KB: all of a compute unit's LDS

#define TRDQ_WIDE_CLOBBERS \
    "v104", "v105", "v106", "v107", "v108", "v109", "v110", "v111", "v112", "v113", "v114", "v115", \
    "v116", "v117", "v118", "v119", "v120", "v121", "v122", "v123", "v124", "v125", "v126", "v127", \
    "v128", "v129", "v130", "v131", "v132", "v133", "v134", "v135", "v136", "v137", "v138", "v139", \
    "v140", "v141", "v142", "v143", "v144", "v145", "v146", "v147", "v148", "v149", "v150", "v151", \
    "v152", "v153", "v154", "v155", "v156", "v157", "v158", "v159", "v160", "v161", "v162", "v163", \
    "v164", "v165", "v166", "v167", "v168", "v169", "v170", "v171", "v172", "v173", "v174", "v175", \
    "v176", "v177", "v178", "v179", "v180", "v181", "v182", "v183", "v184", "v185", "v186", "v187", \
    "v188", "v189", "v190", "v191", "v192", "v193", "v194", "v195", "v196", "v197", "v198", "v199", \
    "v200", "v201", "v202", "v203", "v204", "v205", "v206", "v207", "v208", "v209", "v210", "v211", \
    "v212", "v213", "v214", "v215", "v216", "v217", "v218", "v219", "v220", "v221", "v222", "v223", \
    "v224", "v225", "v226", "v227", "v228", "v229", "v230", "v231", "v232", "v233", "v234", "v235", \
    "v236", "v237", "v238", "v239", "v240", "v241", "v242", "v243", "v244", "v245", "v246", "v247", \
    "v248", "v249", "v250", "v251", "v252", "v253", "v254", "v255", "a0", "a1", "a2", "a3", "a4", \
    "a5", "a6", "a7", "a8", "a9", "a10", "a11", "a12", "a13", "a14", "a15", "a16", "a17", "a18", \
    "a19", "a20", "a21", "a22", "a23", "a24", "a25", "a26", "a27", "a28", "a29", "a30", "a31", \
    "a32", "a33", "a34", "a35", "a36", "a37", "a38", "a39", "a40", "a41", "a42", "a43", "a44", \
    "a45", "a46", "a47", "a48", "a49", "a50", "a51", "a52", "a53", "a54", "a55", "a56", "a57", \
    "a58", "a59", "a60", "a61", "a62", "a63", "a64", "a65", "a66", "a67", "a68", "a69", "a70", \
    "a71", "a72", "a73", "a74", "a75", "a76", "a77", "a78", "a79", "a80", "a81", "a82", "a83", \
    "a84", "a85", "a86", "a87", "a88", "a89", "a90", "a91", "a92", "a93", "a94", "a95", "a96", \
    "a97", "a98", "a99", "a100", "a101", "a102", "a103", "a104", "a105", "a106", "a107", "a108", \
    "a109", "a110", "a111", "a112", "a113", "a114", "a115", "a116", "a117", "a118", "a119", "a120", \
    "a121", "a122", "a123", "a124", "a125", "a126", "a127", "a128", "a129", "a130", "a131", "a132", \
    "a133", "a134", "a135", "a136", "a137", "a138", "a139", "a140", "a141", "a142", "a143", "a144", \
    "a145", "a146", "a147", "a148", "a149", "a150", "a151", "a152", "a153", "a154", "a155", "a156", \
    "a157", "a158", "a159", "a160", "a161", "a162", "a163", "a164", "a165", "a166", "a167", "a168", \
    "a169", "a170", "a171", "a172", "a173", "a174", "a175", "a176", "a177", "a178", "a179", "a180", \
    "a181", "a182", "a183", "a184", "a185", "a186", "a187", "a188", "a189", "a190", "a191", "a192", \
    "a193", "a194", "a195", "a196", "a197", "a198", "a199", "a200", "a201", "a202", "a203", "a204", \
    "a205", "a206", "a207", "a208", "a209", "a210", "a211", "a212", "a213", "a214", "a215", "a216", \
    "a217", "a218", "a219", "a220", "a221", "a222", "a223", "a224", "a225", "a226", "a227", "a228", \
    "a229", "a230", "a231", "a232", "a233", "a234", "a235", "a236", "a237", "a238", "a239", "a240", \
    "a241", "a242", "a243", "a244", "a245", "a246", "a247", "a248", "a249", "a250", "a251", "a252", \
    "a253", "a254", "a255"

template <int... Is, class F>
__device__ __forceinline__ void static_for(std::integer_sequence<int, Is...>, F &&f)
{
    (f(std::integral_constant<int, Is>{}), ...);
}

template <int IDX>
__device__ __forceinline__ int acc_read()
{
    int v;
    asm volatile("v_accvgpr_read_b32 %0, a[%1]" : "=v"(v) : "n"(IDX));
    return v;
}

// LDS ring of five 32 KB slots, one per k-step: row r of an operand at r * 64, its 16-byte
// chunk c at ((c ^ swizzle(r)) * 16).  A copy instruction moves 16 rows x 64 B: lane -> row
// lane / 4, chunk lane % 4 (the LDS side is linear).  Wave w copies rows 64 w .. 64 w + 63 of
// both operands.
//
// Copies are issued for two k-steps at a time: the two 64-byte halves of the same 128-byte
// lines, back to back, into two slots.  Issued a k-step apart, each half costs its own L2
// request (twice the L2-to-L1 traffic); back to back the second half is served by the L1.
//
// Pipeline, k-step s of a tile (fragment set s % 2):
//   wait for the copies of k-step s+1, barrier (slot s is free, slot s+1 is complete), then 64
//   matrix instructions on set s % 2 with, between them, the 16 fragment reads of k-step s+1
//   into the other set and 8 copies: both line halves of four 16-row groups, for k-steps s+4 and
//   s+5 (even s: activation rows) or s+3 and s+4 (odd s: weight rows), into the two slots that
//   the preceding even step found free.  Spreading the copies over all steps matters: the copy
//   unit of a compute unit takes 16 clocks per instruction, and bunched copies stall the waves.
// The copy stream runs on into the next tile of the workgroup; the block ends with vmcnt(0), so
// the next tile's first four k-steps have landed when its block starts.
template <bool DEBUG, bool FULL>
__global__ __launch_bounds__(kThreads) void qgemm8_wide_kernel(GemmArgs g)
{
    extern __shared__ __align__(16) int8_t smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int8_t *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;          // token half, channel half of the wave
    const int l16 = lane & 15, lg = lane >> 4;
    const int K = g.K;
    const int KS = K / kWideBK;                       // k-steps per tile: even, >= 4 (checked by the launcher)
    const int ntiles = g.tiles_m * g.tiles_n;

    // copies: row of this lane inside the tile (first of the wave's 4 instructions; the others
    // are 16 rows apart, which leaves row % 16 and so the swizzle unchanged) and chunk offset
    const int lr = lane >> 2;
    const int rl = wave * 64 + lr;
    const int c0 = ((lane & 3) ^ chunk_swizzle<64>(lr)) * 16;
    // fragment reads: chunk lg of row l16 (+16 rows per fragment)
    const int sw16 = chunk_swizzle<64>(l16);
    const uint32_t xo = lds0 + ((wm * 128 + l16) * 4 + (lg ^ sw16)) * 16;
    const uint32_t wo = lds0 + kWideBM * kWideBK + ((wn * 128 + l16) * 4 + (lg ^ sw16)) * 16;
    const uint32_t wv = lds0 + wave * 4096;

    auto tile_origin = [&](int L, int64_t &m0, int &n0) {
        int tm, tn;
        tile_map(L, g.tiles_m, g.tiles_n, tm, tn);
        m0 = (int64_t)tm * kWideBM;
        n0 = tn * kWideBN;
    };
    auto last_row_x = [&](int64_t m0) { return (int)((g.M - 1 - m0) < 255 ? (g.M - 1 - m0) : 255); };
    auto last_row_w = [&](int n0) { return (g.N - 1 - n0) < 255 ? (g.N - 1 - n0) : 255; };

    int L = blockIdx.x;
    int64_t m0; int n0;
    tile_origin(L, m0, n0);
    int mxc = last_row_x(m0), mwc = last_row_w(n0);
    const int8_t *wbase = static_cast<const int8_t *>(g.Wc);
    uint64_t xp = (uint64_t)(g.Xq + m0 * K);
    uint64_t wp = (uint64_t)(wbase + (int64_t)n0 * K);

    // first four k-steps of the first tile
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rx = (rl + 16 * i) < mxc ? (rl + 16 * i) : mxc;
            dma_1k((uint32_t)(rx * K + c0 + t * kWideBK), (const void *)xp,
                   lds0 + t * kWideSlot + wave * 4096 + i * 1024);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rw = (rl + 16 * i) < mwc ? (rl + 16 * i) : mwc;
            dma_1k((uint32_t)(rw * K + c0 + t * kWideBK), (const void *)wp,
                   lds0 + t * kWideSlot + kWideBM * kWideBK + wave * 4096 + i * 1024);
        }
    }
    wait_vmcnt<0>();

    uint32_t st = 0;                                  // LDS offset of the slot of k-step s
    for (; L < ntiles; L += gridDim.x) {
        const int Ln = L + gridDim.x;
        int64_t m1; int n1;
        tile_origin(Ln < ntiles ? Ln : L, m1, n1);    // after the last tile: re-read it (unused)
        const int mxn = last_row_x(m1), mwn = last_row_w(n1);
        const uint64_t xn = (uint64_t)(g.Xq + m1 * K);
        const uint64_t wnx = (uint64_t)(wbase + (int64_t)n1 * K);

        // Epilogue operands (256 token scales, 256 channel scales, 256 biases): wave w fetches
        // elements 64 w .. 64 w + 63 of each (indices clamped at the matrix edge) at the top of the
        // block and writes them into the ring slot that the last k-step leaves free.
        const int64_t me = m0 + wave * 64 + lane, ne = (int64_t)n0 + wave * 64 + lane;
        const uint32_t vmo = (uint32_t)((me < g.M ? me : g.M - 1) * 4);
        const uint32_t vno = (uint32_t)((ne < g.N ? ne : g.N - 1) * 4);
        const uint64_t sxb = (uint64_t)g.sx, swb = (uint64_t)g.sw, bb = (uint64_t)(g.bias ? g.bias : g.sw);

        uint32_t rem = (uint32_t)__builtin_amdgcn_readfirstlane(KS / 2 - 2);   // pairs of k-steps of this tile still to copy
        uint32_t remw = rem;
        const uint32_t pairs = (uint32_t)__builtin_amdgcn_readfirstlane((KS - 4) / 2);   // k-steps 3 .. KS-2, two per iteration
        uint32_t t0, cnt, sa, sb;
        asm volatile(R"(
  .macro TRDQ_VOFFX maxx, ce
    .irp i,0,1,2,3
      v_add_u32 v126, \i*16, %[rl]
      v_min_u32 v127, \maxx, v126
      v_mad_u32_u24 v[108+\i], v127, %[K], \ce
    .endr
  .endm
  .macro TRDQ_VOFFW maxw, ce
    .irp i,0,1,2,3
      v_add_u32 v126, \i*16, %[rl]
      v_min_u32 v127, \maxw, v126
      v_mad_u32_u24 v[112+\i], v127, %[K], \ce
    .endr
  .endm
  .macro TRDQ_READ set, r, vax, vaw
    .if (\r) < 8
      ds_read_b128 v[128+(\set)*64+(\r)*4:128+(\set)*64+(\r)*4+3], \vaw offset:(\r)*1024
    .else
      ds_read_b128 v[160+(\set)*64+((\r)-8)*4:160+(\set)*64+((\r)-8)*4+3], \vax offset:((\r)-8)*1024
    .endif
  .endm
  ; the copy offsets v108-v115 point at the second 64-byte half of the line; the first half is
  ; reached with the instruction offset -64, which the hardware also adds to the LDS address
  ; (hence the +64 in M0)
  .macro TRDQ_COPY d, half
    .if (\d) < 4
      global_load_lds_dwordx4 v[108+(\d)], %[xp] offset:((\half)-1)*64
    .else
      global_load_lds_dwordx4 v[108+(\d)], %[wp] offset:((\half)-1)*64
    .endif
  .endm
  .macro TRDQ_M0 base, d, half
    .if (\d) < 4
      s_add_u32 m0, \base, (\d)*1024+(1-(\half))*64
    .else
      s_add_u32 m0, \base, 16384+((\d)-4)*1024+(1-(\half))*64
    .endif
  .endm
  .macro TRDQ_STEP set, first, rd, wait, vax, vaw, par=0
    .if \set == 0
      s_cmp_eq_u32 %[rem], 0
      s_cbranch_scc0 .Ltrdq_same\@_%=
      s_mov_b64 %[xp], %[xn]
      TRDQ_VOFFX %[mxn], %[c0]
.Ltrdq_same\@_%=:
      s_sub_u32 %[rem], %[rem], 1
    .else
      s_cmp_eq_u32 %[remw], 0
      s_cbranch_scc0 .Ltrdq_same\@_%=
      s_mov_b64 %[wp], %[wn]
      TRDQ_VOFFW %[mwn], %[c0]
.Ltrdq_same\@_%=:
      s_sub_u32 %[remw], %[remw], 1
    .endif
    s_add_u32 %[t0], %[st], 0x8000
    s_cmp_eq_u32 %[t0], 0x28000
    s_cselect_b32 %[t0], 0, %[t0]
    v_add_u32 \vax, %[t0], %[xo]
    v_add_u32 \vaw, %[t0], %[wo]
    .if \set == 0
      s_sub_u32 %[sa], %[st], 0x8000
      s_cmp_eq_u32 %[st], 0
      s_cselect_b32 %[sa], 0x20000, %[sa]
      s_add_u32 %[sa], %[sa], %[wv]
      s_add_u32 %[sb], %[st], %[wv]
    .endif
    .if \wait
      .if \set == 0
        s_waitcnt vmcnt(16)
      .else
        s_waitcnt vmcnt(8)
      .endif
    .endif
    s_waitcnt lgkmcnt(0)
    s_barrier
    .if \par
      ; this step's slot is free now: it takes the epilogue operands [256 s_x][256 s_w][256 bias]
      v_add_u32 v104, %[st], %[vpo]
      ds_write_b32 v104, v105
      ds_write_b32 v104, v106 offset:1024
      ds_write_b32 v104, v107 offset:2048
    .endif
    .set trdq_n, 0
    .rept 64
      .if \first
        v_mfma_i32_16x16x64_i8 a[trdq_n*4:trdq_n*4+3], v[128+\set*64+(trdq_n/8)*4:128+\set*64+(trdq_n/8)*4+3], v[160+\set*64+(trdq_n%%8)*4:160+\set*64+(trdq_n%%8)*4+3], 0
      .else
        v_mfma_i32_16x16x64_i8 a[trdq_n*4:trdq_n*4+3], v[128+\set*64+(trdq_n/8)*4:128+\set*64+(trdq_n/8)*4+3], v[160+\set*64+(trdq_n%%8)*4:160+\set*64+(trdq_n%%8)*4+3], a[trdq_n*4:trdq_n*4+3]
      .endif
      .if \rd && ((trdq_n %% 2) == 0) && (trdq_n < 32)
        TRDQ_READ 1-\set, trdq_n/2, \vax, \vaw
      .endif
      ; copies: the activation rows' line halves on even steps, the weight rows' on odd steps
      .if (trdq_n %% 16) == 0
        TRDQ_M0 %[sa], (1-\set)*0+\set*4+trdq_n/16, 0
      .endif
      .if (trdq_n %% 16) == 1
        TRDQ_COPY \set*4+trdq_n/16, 0
      .endif
      .if (trdq_n %% 16) == 2
        TRDQ_M0 %[sb], \set*4+trdq_n/16, 1
      .endif
      .if (trdq_n %% 16) == 3
        TRDQ_COPY \set*4+trdq_n/16, 1
      .endif
      .set trdq_n, trdq_n+1
    .endr
    .if \set == 0
      .irp i,108,109,110,111
        v_add_u32 v\i, 0x80, v\i
      .endr
    .else
      .irp i,112,113,114,115
        v_add_u32 v\i, 0x80, v\i
      .endr
    .endif
    s_mov_b32 %[st], %[t0]
  .endm

  ; epilogue operands of this tile, one element of each per lane, parked in v105-v107 until the
  ; last k-step frees a slot for them
  global_load_dword v105, %[vmo], %[sxb]
  global_load_dword v106, %[vno], %[swb]
  global_load_dword v107, %[vno], %[bb]
  TRDQ_VOFFX %[mxc], %[c0e]
  TRDQ_VOFFW %[mwc], %[c0e]
  s_barrier
  v_add_u32 v124, %[st], %[xo]
  v_add_u32 v125, %[st], %[wo]
  .set trdq_r, 0
  .rept 16
    TRDQ_READ 0, trdq_r, v124, v125
    .set trdq_r, trdq_r+1
  .endr
  TRDQ_STEP 0, 1, 1, 0, v122, v123
  TRDQ_STEP 1, 0, 1, 0, v124, v125
  TRDQ_STEP 0, 0, 1, 0, v122, v123
  s_cmp_eq_u32 %[pairs], 0
  s_cbranch_scc1 .Ltrdq_tail_%=
  s_mov_b32 %[cnt], %[pairs]
.Ltrdq_loop_%=:
  TRDQ_STEP 1, 0, 1, 1, v124, v125
  TRDQ_STEP 0, 0, 1, 1, v122, v123
  s_sub_u32 %[cnt], %[cnt], 1
  s_cmp_lg_u32 %[cnt], 0
  s_cbranch_scc1 .Ltrdq_loop_%=
.Ltrdq_tail_%=:
  ; the epilogue operands requested at the top of the block are older than the last 16 copies
  s_waitcnt vmcnt(16)
  TRDQ_STEP 1, 0, 0, 0, v124, v125, 1
  s_waitcnt vmcnt(0) lgkmcnt(0)
  s_barrier
  s_nop 7
  s_nop 7
  .purgem TRDQ_VOFFX
  .purgem TRDQ_VOFFW
  .purgem TRDQ_READ
  .purgem TRDQ_COPY
  .purgem TRDQ_M0
  .purgem TRDQ_STEP
)"
                     // every operand the block writes is early-clobber: an input of equal value
                     // must not share its register
                     : [xp] "+&s"(xp), [wp] "+&s"(wp), [rem] "+&s"(rem), [remw] "+&s"(remw), [st] "+&s"(st), [t0] "=&s"(t0), [cnt] "=&s"(cnt), [sa] "=&s"(sa), [sb] "=&s"(sb)
                     : [xn] "s"(xn), [wn] "s"(wnx),
                       [mxc] "s"(__builtin_amdgcn_readfirstlane(mxc)), [mwc] "s"(__builtin_amdgcn_readfirstlane(mwc)),
                       [mxn] "s"(__builtin_amdgcn_readfirstlane(mxn)), [mwn] "s"(__builtin_amdgcn_readfirstlane(mwn)),
                       [K] "s"(__builtin_amdgcn_readfirstlane(K)), [wv] "s"(__builtin_amdgcn_readfirstlane(wv)),
                       [pairs] "s"(pairs),
                       [sxb] "s"(sxb), [swb] "s"(swb), [bb] "s"(bb), [vmo] "v"(vmo), [vno] "v"(vno),
                       [vpo] "v"(lds0 + (uint32_t)(wave * 256 + lane * 4)),
                       [rl] "v"(rl), [c0] "v"(c0 + 64), [c0e] "v"(c0 + 4 * kWideBK + 64),
                       [xo] "v"(xo), [wo] "v"(wo)
                     : "memory", "scc", "m0", TRDQ_WIDE_CLOBBERS);

        // epilogue: y = float(acc) * s_x[m] * s_w[n] + bias[n] -> bf16.  The lane holds channels
        // n .. n+3 of token m for each of the 8 x 8 instruction tiles; one token tile (16 tokens x
        // 128 channels of the wave) at a time is laid out in the free slot and read back row by
        // row, so that a store instruction writes four whole 256-byte row segments, 16 bytes per
        // lane (partial-line stores reach about half of the store bandwidth).
        const int8_t *const slot = smem + (st == 0 ? 4 * kWideSlot : st - kWideSlot);   // the last k-step's slot
        const float *const par = reinterpret_cast<const float *>(slot);
        constexpr int kRowB = 128 * 2 + 16;                                            // padded staging row
        int8_t *const stg = const_cast<int8_t *>(slot) + 3072 + wave * (16 * kRowB);
        const int64_t m_wave = m0 + wm * 128;
        const int n_wave = n0 + wn * 128;
        const bool has_bias = g.bias != nullptr;
        float4 swv[8], biv[8];
#pragma unroll
        for (int a = 0; a < 8; ++a) {
            swv[a] = *reinterpret_cast<const float4 *>(par + 256 + wn * 128 + a * 16 + lg * 4);
            biv[a] = has_bias ? *reinterpret_cast<const float4 *>(par + 512 + wn * 128 + a * 16 + lg * 4)
                              : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        static_for(std::make_integer_sequence<int, 8>{}, [&](auto bi) {
            constexpr int b = decltype(bi)::value;
            const float sxm = par[wm * 128 + b * 16 + l16];
            static_for(std::make_integer_sequence<int, 8>{}, [&](auto ai) {
                constexpr int a = decltype(ai)::value;
                constexpr int idx = (a * 8 + b) * 4;
                const int q0 = acc_read<idx>(), q1 = acc_read<idx + 1>(), q2 = acc_read<idx + 2>(),
                          q3 = acc_read<idx + 3>();
                if constexpr (DEBUG) {
                    const int64_t m = m_wave + b * 16 + l16;
                    const int n = n_wave + a * 16 + lg * 4;
                    if (FULL || (m < g.M && n < g.N))
                        *reinterpret_cast<int4 *>(g.acc_debug + m * g.N + n) = make_int4(q0, q1, q2, q3);
                }
                uint2 o;
                o.x = pack_bf16x2((float)q0 * sxm * swv[a].x + biv[a].x, (float)q1 * sxm * swv[a].y + biv[a].y);
                o.y = pack_bf16x2((float)q2 * sxm * swv[a].z + biv[a].z, (float)q3 * sxm * swv[a].w + biv[a].w);
                *reinterpret_cast<uint2 *>(stg + l16 * kRowB + (a * 16 + lg * 4) * 2) = o;
            });
            __builtin_amdgcn_wave_barrier();          // compiler: reads below stay after the writes above
            // 16 rows x 256 B = 256 pieces of 16 bytes: four per lane
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int id = i * 64 + lane;
                const int row = id >> 4, c = id & 15;
                const uint4 v = *reinterpret_cast<const uint4 *>(stg + row * kRowB + c * 16);
                const int64_t m = m_wave + b * 16 + row;
                const int n = n_wave + c * 8;
                if (FULL || (m < g.M && n < g.N))
                    store_out16(g.Y + m * g.ldy + n, v);
            }
            __builtin_amdgcn_wave_barrier();          // ... and the next token tile's writes after these reads
        });

        m0 = m1; n0 = n1; mxc = mxn; mwc = mwn;
    }
}

template <bool DEBUG, bool FULL>
hipError_t launch_wide(const GemmArgs &a, hipStream_t st)
{
    GemmArgs g = a;
    g.tiles_m = (int)((g.M + kWideBM - 1) / kWideBM);
    g.tiles_n = (g.N + kWideBN - 1) / kWideBN;
    auto kern = qgemm8_wide_kernel<DEBUG, FULL>;
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), kWideLds); e != hipSuccess) return e;
    int grid = num_cus();
    if (grid > g.tiles_m * g.tiles_n) grid = g.tiles_m * g.tiles_n;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kThreads), kWideLds, st, g);
    return hipGetLastError();
}

}  // namespace

// an even number of k-steps, at least four; 24-bit multiplies form the copy offsets; the output
// is written in 16-byte pieces of 8 channels
bool wide_supports(const GemmArgs &a)
{
    return a.M > 0 && a.K % (2 * kWideBK) == 0 && a.K >= 4 * kWideBK && a.K < (1 << 22) && a.N % 8 == 0 &&
           a.ldy % 8 == 0 && reinterpret_cast<uintptr_t>(a.Y) % 16 == 0;
}

hipError_t launch_qgemm8_wide(const GemmArgs &a, bool debug, hipStream_t st)
{
    if (!wide_supports(a)) return hipErrorInvalidValue;
    const bool full = a.M % kWideBM == 0 && a.N % kWideBN == 0;
    if (debug) return full ? launch_wide<true, true>(a, st) : launch_wide<true, false>(a, st);
    return full ? launch_wide<false, true>(a, st) : launch_wide<false, false>(a, st);
}

}  // namespace gemm
}  // namespace trdq
