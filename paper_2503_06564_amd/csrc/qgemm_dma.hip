// Direct-to-LDS int8 x int8 product kernels for gfx950 (see qgemm.hip for the operand roles).
//
// Tiles travel global -> LDS with global_load_lds_dwordx4: a wave-wide copy moves 64 x 16
// bytes into 1 KB of consecutive LDS, and which global 16-byte chunk a lane fetches is ours
// to choose, so a tile is stored row-major with the chunk index XOR-swizzled by the row
// (conflict-free 16-byte fragment reads, no padding).  The copies are issued from inline
// assembly and tracked by hand: a wave waits with s_waitcnt vmcnt(n) until all but its
// youngest copies have landed, then the workgroup barrier publishes the tile.
//
// Two kernels: `ring` (simple: one barrier per k-tile, fragments read right before use) and
// `pipe` (fragments double-buffered in registers so LDS reads of the next k-step overlap the
// matrix instructions of the current one; one workgroup of four waves per compute unit).
#include "gemm_common.h"

namespace trdq {
namespace gemm {

namespace {

// Dequantising epilogue for int8 weights.  The lane holds, for every 16x16 tile (a, b), the
// accumulators of channels n_lane + 16a .. +3 of token m_lane + 16b:
//   y = float(acc) * s_x[m] * s_w[n] + bias[n]  -> bf16, one 8-byte store per tile.
// FULL: the workgroup tile lies entirely inside the matrix (no bounds checks).
// ASYM: activations carry a zero point; the codes are q - 128 and the integer sum of the product
// of the dequantised operands is acc + (128 - z_m) * colsum[n] (exact in int32).
template <int TN, int TM, bool DEBUG, bool FULL, bool ASYM = false>
__device__ __forceinline__ void epilogue_w8(const v4i (&acc_in)[TN][TM], const GemmArgs &g,
                                            int64_t m_lane, int n_lane)
{
    float sxm[TM];
    int zcm[TM], rsm[TM];
#pragma unroll
    for (int b = 0; b < TM; ++b) {
        const int64_t m = m_lane + b * 16;
        sxm[b] = (FULL || m < g.M) ? g.sx[m] : 0.0f;
        zcm[b] = (ASYM && g.zc && (FULL || m < g.M)) ? g.zc[m] : 0;
        // asymmetric weights: the token's factor of zcw[n] in the zero-point terms
        rsm[b] = (ASYM && g.zcw && (FULL || m < g.M)) ? g.rowsum[m] + g.K * zcm[b] : 0;
    }
    const bool has_bias = g.bias != nullptr;
#pragma unroll
    for (int a = 0; a < TN; ++a) {
        const int n = n_lane + a * 16;
        const bool n_ok = FULL || n < g.N;
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f), bi = s;
        int4 cs = make_int4(0, 0, 0, 0), zw = cs;
        if (n_ok) {
            s = *reinterpret_cast<const float4 *>(g.sw + n);
            if (has_bias) bi = *reinterpret_cast<const float4 *>(g.bias + n);
            if (ASYM) cs = *reinterpret_cast<const int4 *>(g.colsum + n);
            if (ASYM && g.zcw) zw = *reinterpret_cast<const int4 *>(g.zcw + n);
        }
#pragma unroll
        for (int b = 0; b < TM; ++b) {
            const int64_t m = m_lane + b * 16;
            v4i acc[1][1];       // the tile's sums, with the zero-point term when there is one
            acc[0][0] = acc_in[a][b];
            if (ASYM)
                acc[0][0] += v4i{zcm[b] * cs.x + rsm[b] * zw.x, zcm[b] * cs.y + rsm[b] * zw.y,
                                 zcm[b] * cs.z + rsm[b] * zw.z, zcm[b] * cs.w + rsm[b] * zw.w};
            const float y0 = (float)acc[0][0][0] * sxm[b] * s.x + bi.x;
            const float y1 = (float)acc[0][0][1] * sxm[b] * s.y + bi.y;
            const float y2 = (float)acc[0][0][2] * sxm[b] * s.z + bi.z;
            const float y3 = (float)acc[0][0][3] * sxm[b] * s.w + bi.w;
            uint2 o;
            o.x = pack_bf16x2(y0, y1);
            o.y = pack_bf16x2(y2, y3);
            if (FULL || (n_ok && m < g.M)) {
                if constexpr (DEBUG) {
                    int4 d = make_int4(acc[0][0][0], acc[0][0][1], acc[0][0][2], acc[0][0][3]);
                    *reinterpret_cast<int4 *>(g.acc_debug + m * g.N + n) = d;
                }
                *reinterpret_cast<uint2 *>(g.Y + m * g.ldy + n) = o;
            }
        }
    }
}

// Row-wise epilogue for full tiles.  Storing straight from the accumulator layout gives every
// token row 32 contiguous bytes per instruction, and partial-line writes reach only about half
// of the store bandwidth of full lines.  Here each wave first lays its WM x WN block of bf16
// results out in LDS (its own region: no workgroup barrier, LDS serves a wave's requests in
// order), then reads it back row by row, so that one store instruction writes whole
// WN * 2-byte row segments (128 B for a 64-channel wave tile), 16 bytes per lane.
// `stage` is the wave's private LDS region of WM rows of WN * 2 + 16 bytes (the pad spreads the
// column-wise writes over the banks).
// The scales and biases a lane needs in the row-wise epilogue.  Requested before the last k-tile's
// matrix instructions, they arrive while those run instead of stalling the epilogue.
template <int TN, int TM>
struct EpilogueOperands {
    float sxm[TM];
    float4 s[TN], bi[TN];
    __device__ __forceinline__ void load(const GemmArgs &g, int64_t m_wave, int n_wave, int lane)
    {
        const int l16 = lane & 15, lg = lane >> 4;
#pragma unroll
        for (int b = 0; b < TM; ++b) sxm[b] = g.sx[m_wave + b * 16 + l16];
        const bool has_bias = g.bias != nullptr;
#pragma unroll
        for (int a = 0; a < TN; ++a) {
            const int n = n_wave + a * 16 + lg * 4;
            s[a] = *reinterpret_cast<const float4 *>(g.sw + n);
            bi[a] = has_bias ? *reinterpret_cast<const float4 *>(g.bias + n) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
};

template <int TN, int TM, bool DEBUG>
__device__ __forceinline__ void epilogue_w8_rows(const v4i (&acc)[TN][TM], const GemmArgs &g,
                                                 int64_t m_wave, int n_wave, int lane, int8_t *stage,
                                                 const EpilogueOperands<TN, TM> &eo)
{
    constexpr int WN = TN * 16, WM = TM * 16;
    constexpr int ROWB = WN * 2 + 16;
    constexpr int LPR = WN / 8;                  // lanes per row on the way out
    const int l16 = lane & 15, lg = lane >> 4;
    const float (&sxm)[TM] = eo.sxm;
#pragma unroll
    for (int a = 0; a < TN; ++a) {
        const int n = n_wave + a * 16 + lg * 4;
        const float4 s = eo.s[a];
        const float4 bi = eo.bi[a];
#pragma unroll
        for (int b = 0; b < TM; ++b) {
            if constexpr (DEBUG) {
                const int64_t m = m_wave + b * 16 + l16;
                *reinterpret_cast<int4 *>(g.acc_debug + m * g.N + n) =
                    make_int4(acc[a][b][0], acc[a][b][1], acc[a][b][2], acc[a][b][3]);
            }
            const float y0 = (float)acc[a][b][0] * sxm[b] * s.x + bi.x;
            const float y1 = (float)acc[a][b][1] * sxm[b] * s.y + bi.y;
            const float y2 = (float)acc[a][b][2] * sxm[b] * s.z + bi.z;
            const float y3 = (float)acc[a][b][3] * sxm[b] * s.w + bi.w;
            uint2 o;
            o.x = pack_bf16x2(y0, y1);
            o.y = pack_bf16x2(y2, y3);
            *reinterpret_cast<uint2 *>(stage + (b * 16 + l16) * ROWB + (a * 16 + lg * 4) * 2) = o;
        }
    }
    __builtin_amdgcn_wave_barrier();             // compiler: keep the reads below after the writes above
    constexpr int CHUNKS = WM * LPR;             // 16-byte pieces of the block, row-major
#pragma unroll
    for (int i = 0; i < (CHUNKS + 63) / 64; ++i) {
        const int id = i * 64 + lane;
        const int row = id / LPR, c = id % LPR;
        if (CHUNKS % 64 == 0 || id < CHUNKS) {
            const uint4 v = *reinterpret_cast<const uint4 *>(stage + row * ROWB + c * 16);
            store_out16(g.Y + (m_wave + row) * g.ldy + n_wave + c * 8, v);
        }
    }
}

// Zero-point term of asymmetric activations in the pipelined kernels: the accumulators start at
// (128 - z_m) * colsum[n] instead of zero, so the loop and the epilogue are those of the symmetric
// product.  A wave requests its operands (the column sums of its WN channels, 16 bytes per lane,
// and 128 - z of its WM tokens, 4 bytes per lane) as two direct-to-LDS copies into a private block
// of kZpBlock bytes BEFORE the first tile copies; copies retire in order, so the wait for the
// first tile also covers them and the multiplications run while the later tiles are in flight.
// Lanes beyond the slice repeat its last element.  |colsum| < 2^23 (K < 65536) so that the
// products are 24-bit multiplies.
constexpr int kZpBlock = 1024 + 256;

template <int WN, int WM>
__device__ __forceinline__ void zero_point_request(const GemmArgs &g, int64_t m_wave, int n_wave, int lane,
                                                   uint32_t lds_block)
{
    static_assert(WN / 4 <= 64 && WM <= 64, "one copy per operand");
    const uint32_t vc = (uint32_t)((lane < WN / 4 ? lane : WN / 4 - 1) * 16);
    const uint32_t vz = (uint32_t)((lane < WM ? lane : WM - 1) * 4);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(vc), "s"(g.colsum + n_wave), "s"(lds_block) : "memory");
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :: "v"(vz), "s"(g.zc + m_wave), "s"(lds_block + 1024) : "memory");
}

// `on` == 0: plain zeros (the wave group that does not carry the term)
template <int TN, int TM>
__device__ __forceinline__ void zero_point_init(v4i (&acc)[TN][TM], const int8_t *block, int lane, int on)
{
    const int l16 = lane & 15, lg = lane >> 4;
    const int *const b32 = reinterpret_cast<const int *>(block);
    int zcm[TM];
#pragma unroll
    for (int b = 0; b < TM; ++b) zcm[b] = on ? b32[256 + b * 16 + l16] : 0;
#pragma unroll
    for (int a = 0; a < TN; ++a) {
        const int4 c = *reinterpret_cast<const int4 *>(b32 + a * 16 + lg * 4);
#pragma unroll
        for (int b = 0; b < TM; ++b)
            acc[a][b] = v4i{__mul24(zcm[b], c.x), __mul24(zcm[b], c.y), __mul24(zcm[b], c.z), __mul24(zcm[b], c.w)};
    }
}

// Conditional forms whose branch lives inside the assembly block, so that the caller's loop
// body stays one basic block for the compiler (`on` / `steady` are wave-uniform).
__device__ __forceinline__ void dma_1k_if(int on, uint32_t voff, const void *sbase, uint32_t lds_addr)
{
    asm volatile("s_cmp_eq_u32 %3, 0\n\ts_cbranch_scc1 .Lskip%=\n\t"
                 "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n"
                 ".Lskip%=:"
                 :: "v"(voff), "s"(sbase), "s"(lds_addr), "s"(__builtin_amdgcn_readfirstlane(on))
                 : "memory", "scc");
}

// waits for vmcnt(N) when `steady` is set, for vmcnt(0) otherwise
template <int N>
__device__ __forceinline__ void wait_vmcnt_or_zero(int steady)
{
    asm volatile("s_cmp_eq_u32 %0, 0\n\ts_cbranch_scc1 .Lzero%=\n\t"
                 "s_waitcnt vmcnt(%1)\n\ts_branch .Ldone%=\n"
                 ".Lzero%=:\n\ts_waitcnt vmcnt(0)\n"
                 ".Ldone%=:"
                 :: "s"(__builtin_amdgcn_readfirstlane(steady)), "n"(N) : "memory", "scc");
}

template <int BM, int BN, int BK, int NS, int WGM, int WGN, bool DEBUG, bool ASYM = false>
__global__ __launch_bounds__(kThreads) void qgemm8_ring_kernel(GemmArgs g)
{
    static_assert(WGM * WGN == 4, "four waves per workgroup");
    static_assert(BK == 64 || BK == 128, "k-tile of 64 or 128 bytes");
    static_assert(NS >= 3, "at least three stages");
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 16, TN = WN / 16;
    constexpr int CPR = BK / 16;                      // 16-byte chunks per row
    constexpr int XBYTES = BM * BK, WBYTES = BN * BK, STAGE = XBYTES + WBYTES;
    constexpr int PX = XBYTES / 4096, PW = WBYTES / 4096;   // 1 KB copies per wave and tile
    constexpr int P = PX + PW;
    static_assert(PX >= 1 && PW >= 1 && (NS - 2) * P < 64, "copy count per wave out of range");
    constexpr int KH = BK / 64;                       // matrix-instruction k-steps per tile

    extern __shared__ __align__(16) int8_t smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int8_t *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WGM, wn = wave / WGM;
    const int l16 = lane & 15, lg = lane >> 4;

    int tm_idx, tn_idx;
    tile_map(blockIdx.x, g.tiles_m, g.tiles_n, tm_idx, tn_idx);
    const int64_t m0 = (int64_t)tm_idx * BM;
    const int n0 = tn_idx * BN;
    const int K = g.K;

    // ---- copy plan: this lane's source offsets, relative to the tile's first row --------------
    uint32_t voffx[PX], voffw[PW];
#pragma unroll
    for (int i = 0; i < PX; ++i) {
        const int slot = (wave * PX + i) * 64 + lane;
        const int row = slot / CPR, c = (slot % CPR) ^ chunk_swizzle<BK>(row);
        int64_t m = m0 + row;
        if (m >= g.M) m = g.M - 1;                    // rows past M are loaded but never stored
        voffx[i] = (uint32_t)((m - m0) * K + c * 16);
    }
#pragma unroll
    for (int i = 0; i < PW; ++i) {
        const int slot = (wave * PW + i) * 64 + lane;
        const int row = slot / CPR, c = (slot % CPR) ^ chunk_swizzle<BK>(row);
        int n = n0 + row;
        if (n >= g.N) n = g.N - 1;
        voffw[i] = (uint32_t)((n - n0) * K + c * 16);
    }
    const int8_t *xbase = g.Xq + m0 * K;
    const int8_t *wbase = static_cast<const int8_t *>(g.Wc) + (size_t)n0 * K;

    auto issue = [&](int kt, int st) {
        const uint32_t sbase = lds0 + st * STAGE;
#pragma unroll
        for (int i = 0; i < PX; ++i) dma_1k(voffx[i], xbase + kt * BK, sbase + (wave * PX + i) * 1024);
#pragma unroll
        for (int i = 0; i < PW; ++i) dma_1k(voffw[i], wbase + kt * BK, sbase + XBYTES + (wave * PW + i) * 1024);
    };

    // ---- fragment read offsets inside a stage ----------------------------------------------------
    int xoff[KH], woff[KH];
#pragma unroll
    for (int h = 0; h < KH; ++h) {
        const int pc = (4 * h + lg) ^ chunk_swizzle<BK>(l16);
        xoff[h] = ((wm * WM + l16) * CPR + pc) * 16;
        woff[h] = XBYTES + ((wn * WN + l16) * CPR + pc) * 16;
    }

    v4i acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b) acc[a][b] = v4i{0, 0, 0, 0};

    const int KT = K / BK;
#pragma unroll
    for (int t = 0; t < NS - 1; ++t)
        if (t < KT) issue(t, t);

    int st = 0;
    for (int kt = 0; kt < KT; ++kt) {
        if (kt + NS - 1 <= KT) wait_vmcnt<(NS - 2) * P>();
        else wait_vmcnt<0>();
        __syncthreads();
        if (kt + NS - 1 < KT) issue(kt + NS - 1, st == 0 ? NS - 1 : st - 1);

        const int8_t *stage = smem + st * STAGE;
#pragma unroll
        for (int h = 0; h < KH; ++h) {
            v4i af[TN], bf[TM];
#pragma unroll
            for (int a = 0; a < TN; ++a) af[a] = *reinterpret_cast<const v4i *>(stage + woff[h] + a * 16 * BK);
#pragma unroll
            for (int b = 0; b < TM; ++b) bf[b] = *reinterpret_cast<const v4i *>(stage + xoff[h] + b * 16 * BK);
#pragma unroll
            for (int a = 0; a < TN; ++a)
#pragma unroll
                for (int b = 0; b < TM; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[a], bf[b], acc[a][b], 0, 0, 0);
        }
        st = (st + 1 == NS) ? 0 : st + 1;
    }

    epilogue_w8<TN, TM, DEBUG, false, ASYM>(acc, g, m0 + wm * WM + l16, n0 + wn * WN + lg * 4);
}

// ---- software-pipelined kernel ---------------------------------------------------------------
template <int TN, int TM, int BK>
__device__ __forceinline__ void load_frags(v4i (&af)[TN], v4i (&bf)[TM], const int8_t *stage, int woff, int xoff)
{
#pragma unroll
    for (int a = 0; a < TN; ++a) af[a] = *reinterpret_cast<const v4i *>(stage + woff + a * 16 * BK);
#pragma unroll
    for (int b = 0; b < TM; ++b) bf[b] = *reinterpret_cast<const v4i *>(stage + xoff + b * 16 * BK);
}

template <int TN, int TM>
__device__ __forceinline__ void mfma_block(v4i (&acc)[TN][TM], const v4i (&af)[TN], const v4i (&bf)[TM])
{
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
            acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[a], bf[b], acc[a][b], 0, 0, 0);
}

// Ask the scheduler to issue the NREAD LDS reads of the next step early: one read in front of
// each of the first matrix instructions of the current step, the remaining matrix instructions
// after them, so the fragments have the rest of the step to arrive.
template <int NREAD, int NMFMA>
__device__ __forceinline__ void interleave_hint()
{
    constexpr int LEAD = NREAD < NMFMA ? NREAD : NMFMA;
#pragma unroll
    for (int i = 0; i < LEAD; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // one LDS read
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one matrix instruction
    }
    if constexpr (NREAD > LEAD) __builtin_amdgcn_sched_group_barrier(0x100, NREAD - LEAD, 0);
    if constexpr (NMFMA > LEAD) __builtin_amdgcn_sched_group_barrier(0x008, NMFMA - LEAD, 0);
}

// BK = 128: two matrix-instruction k-steps per tile.  Fragment set F0 serves step 0 and F1
// step 1; while one feeds the matrix cores the other is being filled.  At the end of tile kt
// the workgroup waits for tile kt+1, passes the barrier (which also retires every read of
// tile kt's stage), refills that stage with tile kt+NS and starts reading tile kt+1.
template <int BM, int BN, int NS, int WGM, int WGN, bool DEBUG, bool ASYM = false>
__global__ __launch_bounds__(WGM * WGN * 64) void qgemm8_pipe_kernel(GemmArgs g)
{
    constexpr int NW = WGM * WGN;                     // waves per workgroup
    static_assert(NW == 4 || NW == 8, "four or eight waves per workgroup");
    static_assert(NS >= 2, "at least two stages");
    constexpr int BK = 128;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 16, TN = WN / 16;
    constexpr int CPR = BK / 16;
    // weight rows are copied 8 at a time; a channel count that does not split evenly over the
    // waves (BN = 144: 18 copies) is rounded up, the surplus copies repeat the last rows
    // into LDS space nobody reads
    constexpr int WG8 = BN / 8;                       // 8-row groups of weight rows
    constexpr int XBYTES = BM * BK;
    constexpr int PX = XBYTES / (NW * 1024), PW = (WG8 + NW - 1) / NW;
    constexpr int WBYTES = NW * PW * 1024, STAGE = XBYTES + WBYTES;
    constexpr int P = PX + PW;
    static_assert(BN % 16 == 0 && PX >= 1 && PX % 2 == 0 && (NS - 1) * P < 64, "copy count per wave out of range");

    extern __shared__ __align__(16) int8_t smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int8_t *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WGM, wn = wave / WGM;
    const int l16 = lane & 15, lg = lane >> 4;

    int tm_idx, tn_idx;
    tile_map(blockIdx.x, g.tiles_m, g.tiles_n, tm_idx, tn_idx);
    const int64_t m0 = (int64_t)tm_idx * BM;
    const int n0 = tn_idx * BN;
    const int K = g.K;

    // Copy plan (tiles are full: M % BM == 0 and N % BN == 0 on this path).  Copy i of a wave
    // fills LDS rows (wave*PX + i)*8 .. +7, eight 16-byte chunks each; the lane's row inside
    // the 16-row swizzle period only depends on the parity of i, so two lane offsets per
    // operand are enough and the rest of the address is scalar.
    uint32_t voff[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int r = 8 * p + (lane >> 3);
        voff[p] = (uint32_t)(r * K + (((lane & 7) ^ chunk_swizzle<BK>(r)) * 16));
    }
    const int8_t *xbase = g.Xq + (m0 + wave * PX * 8) * K;
    const int8_t *wbase = static_cast<const int8_t *>(g.Wc) + (size_t)n0 * K;
    const int K16 = 16 * K;
    // weight copy i of this wave: 8-row group j = wave * PW + i (clamped to the last group)
    uint32_t voffw[PW];
    int wrow[PW];
#pragma unroll
    for (int i = 0; i < PW; ++i) {
        int j = wave * PW + i;
        if (j > WG8 - 1) j = WG8 - 1;
        voffw[i] = voff[j & 1];
        wrow[i] = __builtin_amdgcn_readfirstlane((j & ~1) * 8);
    }

    auto issue = [&](int on, int kt, int st) {
        const uint32_t sbase = lds0 + st * STAGE;
        const int8_t *xs = xbase + kt * BK, *ws = wbase + kt * BK;
#pragma unroll
        for (int i = 0; i < PX; ++i)
            dma_1k_if(on, voff[i & 1], xs + (i >> 1) * K16, sbase + (wave * PX + i) * 1024);
#pragma unroll
        for (int i = 0; i < PW; ++i)
            dma_1k_if(on, voffw[i], ws + wrow[i] * K, sbase + XBYTES + (wave * PW + i) * 1024);
    };

    int xoff[2], woff[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int pc = (4 * h + lg) ^ chunk_swizzle<BK>(l16);
        xoff[h] = ((wm * WM + l16) * CPR + pc) * 16;
        woff[h] = XBYTES + ((wn * WN + l16) * CPR + pc) * 16;
    }

    v4i acc[TN][TM];
    v4i af0[TN], bf0[TM], af1[TN], bf1[TM];

    const int KT = K / BK;
    if constexpr (ASYM) zero_point_request<WN, WM>(g, m0 + wm * WM, n0 + wn * WN, lane, lds0 + NS * STAGE + wave * kZpBlock);
#pragma unroll
    for (int t = 0; t < NS; ++t) issue(t < KT, t, t);
    wait_vmcnt_or_zero<(NS - 1) * P>(KT >= NS);
    __syncthreads();
    if constexpr (ASYM) {
        zero_point_init<TN, TM>(acc, smem + NS * STAGE + wave * kZpBlock, lane, 1);
    } else {
#pragma unroll
        for (int a = 0; a < TN; ++a)
#pragma unroll
            for (int b = 0; b < TM; ++b) acc[a][b] = v4i{0, 0, 0, 0};
    }
    load_frags<TN, TM, BK>(af0, bf0, smem, woff[0], xoff[0]);

    // The loop body is straight-line code (the conditional copy and wait branch inside their
    // assembly blocks), which keeps the accumulators in place across iterations.
    int st = 0;
    for (int kt = 0; kt + 1 < KT; ++kt) {
        const int nst = (st + 1 == NS) ? 0 : st + 1;
        const int more = kt + NS < KT;       // tile kt+NS exists and replaces tile kt in its stage
        load_frags<TN, TM, BK>(af1, bf1, smem + st * STAGE, woff[1], xoff[1]);
        mfma_block<TN, TM>(acc, af0, bf0);
        interleave_hint<TN + TM, TN * TM>();
        wait_vmcnt_or_zero<(NS - 2) * P>(more);   // tile kt+1 has landed (this wave's share)
        __syncthreads();                          // ... everyone's share; tile kt's stage is retired
        issue(more, kt + NS, st);
        load_frags<TN, TM, BK>(af0, bf0, smem + nst * STAGE, woff[0], xoff[0]);
        mfma_block<TN, TM>(acc, af1, bf1);
        interleave_hint<TN + TM, TN * TM>();
        st = nst;
    }
    // last tile (every copy has landed: ordinary loads no longer queue behind them)
    constexpr bool kRowsEpilogue = NW * WM * (WN * 2 + 16) <= NS * STAGE;
    EpilogueOperands<TN, TM> eo;
    if constexpr (kRowsEpilogue) eo.load(g, m0 + wm * WM, n0 + wn * WN, lane);
    load_frags<TN, TM, BK>(af1, bf1, smem + st * STAGE, woff[1], xoff[1]);
    mfma_block<TN, TM>(acc, af0, bf0);
    interleave_hint<TN + TM, TN * TM>();
    mfma_block<TN, TM>(acc, af1, bf1);

    if constexpr (kRowsEpilogue) {
        // every wave is done with the ring: reuse it as the epilogue's staging space
        __syncthreads();
        epilogue_w8_rows<TN, TM, DEBUG>(acc, g, m0 + wm * WM, n0 + wn * WN, lane, smem + wave * (WM * (WN * 2 + 16)), eo);
    } else {
        epilogue_w8<TN, TM, DEBUG, true>(acc, g, m0 + wm * WM + l16, n0 + wn * WN + lg * 4);
    }
}

// ---- software-pipelined kernel, two wave groups splitting K inside the workgroup ----------------
// Same tile and pipeline as qgemm8_pipe_kernel, but with eight waves: waves 0-3 accumulate the
// first half of the k-tiles, waves 4-7 the second half, each group on its own ring of NS stages;
// at the end the groups swap halves of their sums through LDS and each finishes the token rows
// of one half (the first group takes one k-tile more when their number is odd; the second then
// sits out the last step, so that both meet at the same barriers).  For a launch of one tile per compute unit (few tokens, long K) this puts two
// independent instruction streams on every SIMD, which overlap each other's copy issue, LDS reads
// and barriers the way a second resident workgroup would, without a second tile to give it.
// Needs at least NS k-tiles per group.
template <int BM, int BN, int NS, int WGM, int WGN, bool DEBUG, bool ASYM = false>
__global__ __launch_bounds__(2 * kThreads) void qgemm8_pipe2_kernel(GemmArgs g)
{
    static_assert(WGM * WGN == 4, "four waves per group");
    static_assert(NS >= 2, "at least two stages");
    constexpr int BK = 128;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 16, TN = WN / 16;
    constexpr int CPR = BK / 16;
    constexpr int WG8 = BN / 8;
    constexpr int XBYTES = BM * BK;
    constexpr int PX = XBYTES / 4096, PW = (WG8 + 3) / 4;
    constexpr int WBYTES = 4 * PW * 1024, STAGE = XBYTES + WBYTES;
    constexpr int P = PX + PW;
    constexpr int RING = NS * STAGE;
    static_assert(BN % 16 == 0 && PX >= 1 && PX % 2 == 0 && (NS - 1) * P < 64, "copy count per wave out of range");
    static_assert(TM % 2 == 0, "each group finishes half of the token tiles");
    constexpr int TMH = TM / 2;
    constexpr int XCH = TN * TMH * 256 * 16;         // bytes of the sums one group hands over
    constexpr int STG = 16 * TMH * (WN * 2 + 16);    // a wave's staging block in the epilogue
    static_assert(XCH + 4 * STG <= RING, "hand-over area and epilogue staging must fit a group's ring");

    extern __shared__ __align__(16) int8_t smem[];

    const int tid = threadIdx.x & 255;
    const int lane = tid & 63;
    const int kg = __builtin_amdgcn_readfirstlane(threadIdx.x >> 8);      // wave group: which half of K
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WGM, wn = wave / WGM;
    const int l16 = lane & 15, lg = lane >> 4;
    int8_t *const ring = smem + kg * RING;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int8_t *)ring;

    int tm_idx, tn_idx;
    tile_map(blockIdx.x, g.tiles_m, g.tiles_n, tm_idx, tn_idx);
    const int64_t m0 = (int64_t)tm_idx * BM;
    const int n0 = tn_idx * BN;
    const int K = g.K;
    const int KTA = K / BK;                          // k-tiles of the product
    const int KTX = (KTA + 1) / 2;                   // steps of both groups = k-tiles of the first
    const int KT = kg == 0 ? KTX : KTA - KTX;        // this group's k-tiles
    const int kofs = kg * KTX * BK;                  // this group's first k

    uint32_t voff[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int r = 8 * p + (lane >> 3);
        voff[p] = (uint32_t)(r * K + (((lane & 7) ^ chunk_swizzle<BK>(r)) * 16));
    }
    const int8_t *xbase = g.Xq + (m0 + wave * PX * 8) * K + kofs;
    const int8_t *wbase = static_cast<const int8_t *>(g.Wc) + (size_t)n0 * K + kofs;
    const int K16 = 16 * K;
    uint32_t voffw[PW];
    int wrow[PW];
#pragma unroll
    for (int i = 0; i < PW; ++i) {
        int j = wave * PW + i;
        if (j > WG8 - 1) j = WG8 - 1;
        voffw[i] = voff[j & 1];
        wrow[i] = __builtin_amdgcn_readfirstlane((j & ~1) * 8);
    }

    auto issue = [&](int on, int kt, int st) {
        const uint32_t sbase = lds0 + st * STAGE;
        const int8_t *xs = xbase + kt * BK, *ws = wbase + kt * BK;
#pragma unroll
        for (int i = 0; i < PX; ++i)
            dma_1k_if(on, voff[i & 1], xs + (i >> 1) * K16, sbase + (wave * PX + i) * 1024);
#pragma unroll
        for (int i = 0; i < PW; ++i)
            dma_1k_if(on, voffw[i], ws + wrow[i] * K, sbase + XBYTES + (wave * PW + i) * 1024);
    };

    int xoff[2], woff[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int pc = (4 * h + lg) ^ chunk_swizzle<BK>(l16);
        xoff[h] = ((wm * WM + l16) * CPR + pc) * 16;
        woff[h] = XBYTES + ((wn * WN + l16) * CPR + pc) * 16;
    }

    v4i acc[TN][TM];
    v4i af0[TN], bf0[TM], af1[TN], bf1[TM];

    // asymmetric activations: both groups request the operands (same copy counts), the first carries the term
    const int zblock = 2 * RING + (kg * 4 + wave) * kZpBlock;
    if constexpr (ASYM)
        zero_point_request<WN, WM>(g, m0 + wm * WM, n0 + wn * WN, lane,
                                   (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int8_t *)smem + zblock);
#pragma unroll
    for (int t = 0; t < NS; ++t) issue(t < KT, t, t);
    wait_vmcnt_or_zero<(NS - 1) * P>(KT >= NS);
    __syncthreads();
    if constexpr (ASYM) {
        zero_point_init<TN, TM>(acc, smem + zblock, lane, kg == 0);
    } else {
#pragma unroll
        for (int a = 0; a < TN; ++a)
#pragma unroll
            for (int b = 0; b < TM; ++b) acc[a][b] = v4i{0, 0, 0, 0};
    }
    load_frags<TN, TM, BK>(af0, bf0, ring, woff[0], xoff[0]);

    // both groups run the same number of iterations, so they meet at the same barriers
    int st = 0;
    for (int kt = 0; kt + 1 < KTX; ++kt) {
        const int nst = (st + 1 == NS) ? 0 : st + 1;
        const int more = kt + NS < KT;
        load_frags<TN, TM, BK>(af1, bf1, ring + st * STAGE, woff[1], xoff[1]);
        mfma_block<TN, TM>(acc, af0, bf0);
        interleave_hint<TN + TM, TN * TM>();
        wait_vmcnt_or_zero<(NS - 2) * P>(more);
        __syncthreads();
        issue(more, kt + NS, st);
        load_frags<TN, TM, BK>(af0, bf0, ring + nst * STAGE, woff[0], xoff[0]);
        mfma_block<TN, TM>(acc, af1, bf1);
        interleave_hint<TN + TM, TN * TM>();
        st = nst;
    }
    // last step (the second group has no tile left here when the count is odd)
    const int64_t m_own = m0 + wm * WM + kg * TMH * 16;      // token rows this group finishes
    EpilogueOperands<TN, TMH> eo;
    eo.load(g, m_own, n0 + wn * WN, lane);
    if (KT == KTX) {
        load_frags<TN, TM, BK>(af1, bf1, ring + st * STAGE, woff[1], xoff[1]);
        mfma_block<TN, TM>(acc, af0, bf0);
        interleave_hint<TN + TM, TN * TM>();
        mfma_block<TN, TM>(acc, af1, bf1);
    }

    // Hand-over.  Both rings are free once every wave has read its last fragments.  Each group
    // writes the sums of the token tiles it does not finish into the other group's ring (one
    // 16-byte piece per lane and accumulator tile), then adds what it received to its own half.
    __syncthreads();
    {
        v4i *const out = reinterpret_cast<v4i *>(smem + (1 - kg) * RING);
#pragma unroll
        for (int a = 0; a < TN; ++a)
#pragma unroll
            for (int b = 0; b < TMH; ++b) {
                if (kg == 0) out[(a * TMH + b) * 256 + tid] = acc[a][TMH + b];     // register indices stay static
                else out[(a * TMH + b) * 256 + tid] = acc[a][b];
            }
    }
    __syncthreads();
    v4i own[TN][TMH];
    {
        const v4i *const in = reinterpret_cast<const v4i *>(ring);
#pragma unroll
        for (int a = 0; a < TN; ++a)
#pragma unroll
            for (int b = 0; b < TMH; ++b) {
                const v4i o = in[(a * TMH + b) * 256 + tid];
                own[a][b] = (kg == 0 ? acc[a][b] : acc[a][TMH + b]) + o;
            }
    }
    epilogue_w8_rows<TN, TMH, DEBUG>(own, g, m_own, n0 + wn * WN, lane, ring + XCH + wave * STG, eo);
}

// ---- persistent software-pipelined kernel -------------------------------------------------------
// A workgroup walks a list of output tiles.  The k-tile ring never drains between tiles: while
// the last k-tiles of tile T are multiplied, the first k-tiles of tile T+1 are already being
// copied, the epilogue's stores overlap the next tile's main loop, and a second workgroup on
// the same compute unit fills the matrix cores while this one converts and stores.

// waits for vmcnt(NBIG) / vmcnt(N) / vmcnt(0) for sel = 2 / 1 / 0 (sel is wave-uniform)
template <int N, int NBIG>
__device__ __forceinline__ void wait_vmcnt_select(int sel)
{
    asm volatile("s_cmp_eq_u32 %0, 2\n\ts_cbranch_scc0 .Lnotbig%=\n\t"
                 "s_waitcnt vmcnt(%2)\n\ts_branch .Ldone%=\n"
                 ".Lnotbig%=:\n\ts_cmp_eq_u32 %0, 1\n\ts_cbranch_scc0 .Lzero%=\n\t"
                 "s_waitcnt vmcnt(%1)\n\ts_branch .Ldone%=\n"
                 ".Lzero%=:\n\ts_waitcnt vmcnt(0)\n"
                 ".Ldone%=:"
                 :: "s"(__builtin_amdgcn_readfirstlane(sel)), "n"(N), "n"(NBIG) : "memory", "scc");
}

template <int BM, int BN, int NS, int WGM, int WGN, bool DEBUG>
__global__ __launch_bounds__(kThreads) void qgemm8_persist_kernel(GemmArgs g)
{
    static_assert(WGM * WGN == 4, "four waves per workgroup");
    static_assert(NS >= 2, "at least two stages");
    constexpr int BK = 128;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 16, TN = WN / 16;
    constexpr int CPR = BK / 16;
    constexpr int XBYTES = BM * BK, WBYTES = BN * BK, STAGE = XBYTES + WBYTES;
    constexpr int PX = XBYTES / 4096, PW = WBYTES / 4096;
    constexpr int P = PX + PW;
    constexpr int SEP = TN * TM * (DEBUG ? 2 : 1);                    // store instructions of one epilogue
    constexpr int NWAIT = (NS - 2) * P;
    constexpr int NBIG = NWAIT + SEP < 63 ? NWAIT + SEP : 63;
    static_assert(PX % 2 == 0 && PW % 2 == 0 && (NS - 1) * P < 64, "copy counts");

    extern __shared__ __align__(16) int8_t smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int8_t *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WGM, wn = wave / WGM;
    const int l16 = lane & 15, lg = lane >> 4;
    const int K = g.K;
    const int KT = K / BK;                            // >= NS (checked by the launcher)
    const int ntiles = g.tiles_m * g.tiles_n;

    uint32_t voff[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int r = 8 * p + (lane >> 3);
        voff[p] = (uint32_t)(r * K + (((lane & 7) ^ chunk_swizzle<BK>(r)) * 16));
    }
    const int K16 = 16 * K;
    int xoff[2], woff[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int pc = (4 * h + lg) ^ chunk_swizzle<BK>(l16);
        xoff[h] = ((wm * WM + l16) * CPR + pc) * 16;
        woff[h] = XBYTES + ((wn * WN + l16) * CPR + pc) * 16;
    }

    // tile id -> operand bases of this wave's copies
    auto tile_coords = [&](int L, int64_t &m0, int &n0) {
        int tm, tn;
        tile_map(L, g.tiles_m, g.tiles_n, tm, tn);
        m0 = (int64_t)tm * BM;
        n0 = tn * BN;
    };
    // Copies are unconditional: past the workgroup's last tile they re-read that tile's own
    // k-tiles into stages nobody reads any more (a few redundant cached reads at the very end)
    // instead of branching around every copy.
    auto issue = [&](const int8_t *xs, const int8_t *ws, int st) {
        const uint32_t sbase = lds0 + st * STAGE;
#pragma unroll
        for (int i = 0; i < PX; ++i)
            dma_1k(voff[i & 1], xs + (i >> 1) * K16, sbase + (wave * PX + i) * 1024);
#pragma unroll
        for (int i = 0; i < PW; ++i)
            dma_1k(voff[i & 1], ws + (i >> 1) * K16, sbase + XBYTES + (wave * PW + i) * 1024);
    };

    int L = blockIdx.x;                               // this workgroup's tiles: L, L + grid, ...
    int64_t m0; int n0;
    tile_coords(L, m0, n0);
    const int8_t *xcur = g.Xq + (m0 + wave * PX * 8) * K;
    const int8_t *wcur = static_cast<const int8_t *>(g.Wc) + ((size_t)n0 + wave * PW * 8) * K;

#pragma unroll
    for (int t = 0; t < NS; ++t) issue(xcur + t * BK, wcur + t * BK, t);
    wait_vmcnt<(NS - 1) * P>();
    __syncthreads();
    v4i af0[TN], bf0[TM], af1[TN], bf1[TM];
    load_frags<TN, TM, BK>(af0, bf0, smem, woff[0], xoff[0]);

    int st = 0;
    bool first = true;
    for (; L < ntiles; L += gridDim.x) {
        // next tile of this workgroup (its first k-tiles are prefetched during this tile's last ones)
        const int Ln = L + gridDim.x;
        const int has_next = Ln < ntiles;
        int64_t m1 = 0; int n1 = 0;
        tile_coords(has_next ? Ln : L, m1, n1);
        const int8_t *xnext = g.Xq + (m1 + wave * PX * 8) * K;
        const int8_t *wnext = static_cast<const int8_t *>(g.Wc) + ((size_t)n1 + wave * PW * 8) * K;

        const int64_t m_lane = m0 + wm * WM + l16;
        const int n_lane = n0 + wn * WN + lg * 4;

        v4i acc[TN][TM];
#pragma unroll
        for (int a = 0; a < TN; ++a)
#pragma unroll
            for (int b = 0; b < TM; ++b) acc[a][b] = v4i{0, 0, 0, 0};

        for (int kt = 0; kt < KT; ++kt) {
            const int nst = (st + 1 == NS) ? 0 : st + 1;
            // the copy issued in this step is k-tile kt + NS of this tile, or wraps into the next
            // tile (after the last tile: into this tile again, unused)
            const int wrap = kt + NS >= KT;
            const int ikt = wrap ? kt + NS - KT : kt + NS;
            const int8_t *xs = (wrap ? xnext : xcur) + ikt * BK;
            const int8_t *ws = (wrap ? wnext : wcur) + ikt * BK;
            // younger than the k-tile waited for: (NS-2) k-tiles of copies, plus -- in the first
            // NS-1 steps after an epilogue -- that epilogue's stores
            const int sel = (!first && kt < NS - 1) ? 2 : 1;

            load_frags<TN, TM, BK>(af1, bf1, smem + st * STAGE, woff[1], xoff[1]);
            mfma_block<TN, TM>(acc, af0, bf0);
            interleave_hint<TN + TM, TN * TM>();
            wait_vmcnt_select<NWAIT, NBIG>(sel);
            __syncthreads();
            issue(xs, ws, st);
            load_frags<TN, TM, BK>(af0, bf0, smem + nst * STAGE, woff[0], xoff[0]);
            mfma_block<TN, TM>(acc, af1, bf1);
            interleave_hint<TN + TM, TN * TM>();
            st = nst;
        }

        // epilogue (full tiles only on this path): y = float(acc) * s_x * s_w + bias -> bf16.
        // Its operands are ordinary loads: the compiler's own wait for them also covers the
        // copies already requested for the next tile, which costs a little overlap and keeps
        // every register the loads write under the compiler's control.
        float sxm[TM];
        float4 swv[TN], biv[TN];
#pragma unroll
        for (int b = 0; b < TM; ++b) sxm[b] = g.sx[m_lane + b * 16];
#pragma unroll
        for (int a = 0; a < TN; ++a) {
            swv[a] = *reinterpret_cast<const float4 *>(g.sw + n_lane + a * 16);
            biv[a] = g.bias ? *reinterpret_cast<const float4 *>(g.bias + n_lane + a * 16) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int a = 0; a < TN; ++a) {
            const int n = n_lane + a * 16;
#pragma unroll
            for (int b = 0; b < TM; ++b) {
                const int64_t m = m_lane + b * 16;
                if constexpr (DEBUG) {
                    int4 d = make_int4(acc[a][b][0], acc[a][b][1], acc[a][b][2], acc[a][b][3]);
                    *reinterpret_cast<int4 *>(g.acc_debug + m * g.N + n) = d;
                }
                const float y0 = (float)acc[a][b][0] * sxm[b] * swv[a].x + biv[a].x;
                const float y1 = (float)acc[a][b][1] * sxm[b] * swv[a].y + biv[a].y;
                const float y2 = (float)acc[a][b][2] * sxm[b] * swv[a].z + biv[a].z;
                const float y3 = (float)acc[a][b][3] * sxm[b] * swv[a].w + biv[a].w;
                uint2 o;
                o.x = pack_bf16x2(y0, y1);
                o.y = pack_bf16x2(y2, y3);
                *reinterpret_cast<uint2 *>(g.Y + m * g.ldy + n) = o;
            }
        }
        m0 = m1; n0 = n1; xcur = xnext; wcur = wnext;
        first = false;
    }
}

// ---- int4 weights on the direct-to-LDS path --------------------------------------------------------
// Activations as in the int8 kernels (128-byte k-tiles, 8 rows per copy).  A weight row of a
// k-tile is 64 packed bytes (one 128-channel scale group), 16 rows per copy; the lane reads the
// 8 packed bytes of its 16 codes and widens them in registers to 16 * code (nibble moved to the
// top of the byte: one shift-and-mask and one mask per 8 codes).  At the end of every k-tile the
// int32 sums of the group are folded into float accumulators with the group's scales
// (Eq. 1 per 128-input group); the factor 16 is undone with the token scale in the epilogue.
//
// The group's 128 scales travel with the k-tile: one more direct-to-LDS copy per wave (4 bytes
// per lane; waves 2 and 3 write a second, unused copy so that every wave issues the same number
// of requests and the hand-kept vmcnt arithmetic stays uniform).  Past the last k-tile the last
// one is copied again, for the same reason.
// ASYM: asymmetric activations (codes q - 128, zc = 128 - z per token).  The zero-point term of group g
// is zc * colsum_g[n]; scaled and summed over the groups it is zc * cw[n] with the per-channel float
// cw[n] = 16 * sum_g s_w[g][n] * colsum_g[n] prepared with the weights, so it costs one multiply-add
// per output in the epilogue.
template <int BM, int BN, int NS, int WGM, int WGN, bool DEBUG, bool ASYM = false>
__global__ __launch_bounds__(kThreads) void qgemm4_ring_kernel(GemmArgs g)
{
    static_assert(WGM * WGN == 4, "four waves per workgroup");
    static_assert(NS >= 2, "at least two stages");
    constexpr int BK = 128;                           // = one int4 scale group
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 16, TN = WN / 16;
    constexpr int XBYTES = BM * BK, WBYTES = BN * (BK / 2), SOFF = XBYTES + WBYTES;
    constexpr int STAGE = SOFF + 1024;                // + [2][BN] scales
    constexpr int PX = XBYTES / 4096, PW = WBYTES / 4096;
    constexpr int P = PX + PW + 1;                    // copies per wave and k-tile
    static_assert(BN == 128, "one scale copy of 64 lanes per channel half");
    static_assert(PX >= 1 && PW >= 1 && (NS - 2) * P < 64, "request counts");

    extern __shared__ __align__(16) int8_t smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int8_t *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WGM, wn = wave / WGM;
    const int l16 = lane & 15, lg = lane >> 4;

    int tm_idx, tn_idx;
    tile_map(blockIdx.x, g.tiles_m, g.tiles_n, tm_idx, tn_idx);
    const int64_t m0 = (int64_t)tm_idx * BM;
    const int n0 = tn_idx * BN;
    const int K = g.K;
    const int KT = K / BK;

    // copy plan (rows past the matrix edge are clamped: loaded, never stored)
    uint32_t voffx[PX], voffw[PW];
#pragma unroll
    for (int i = 0; i < PX; ++i) {
        const int slot = (wave * PX + i) * 64 + lane;
        const int row = slot / 8, c = (slot % 8) ^ chunk_swizzle<128>(row);
        int64_t m = m0 + row;
        if (m >= g.M) m = g.M - 1;
        voffx[i] = (uint32_t)((m - m0) * K + c * 16);
    }
#pragma unroll
    for (int i = 0; i < PW; ++i) {
        const int slot = (wave * PW + i) * 64 + lane;
        const int row = slot / 4, c = (slot % 4) ^ ((row >> 2) & 3);   // 64-byte rows: spread rows r, r+4, r+8, r+12
        int n = n0 + row;
        if (n >= g.N) n = g.N - 1;
        voffw[i] = (uint32_t)((n - n0) * (K / 2) + c * 16);
    }
    int ns = n0 + (wave & 1) * 64 + lane;
    if (ns >= g.N) ns = g.N - 1;
    const uint32_t voffs = (uint32_t)((ns - n0) * 4);
    const int8_t *xbase = g.Xq + m0 * K;
    const uint8_t *wbase = static_cast<const uint8_t *>(g.Wc) + (size_t)n0 * (K / 2);
    const float *sbase_g = g.sw + n0;
    auto issue = [&](int kt, int st) {
        const uint32_t sbase = lds0 + st * STAGE;
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                     :: "v"(voffs), "s"(sbase_g + (size_t)kt * g.N), "s"(sbase + SOFF + wave * 256) : "memory");
#pragma unroll
        for (int i = 0; i < PX; ++i) dma_1k(voffx[i], xbase + kt * BK, sbase + (wave * PX + i) * 1024);
#pragma unroll
        for (int i = 0; i < PW; ++i) dma_1k(voffw[i], wbase + kt * (BK / 2), sbase + XBYTES + (wave * PW + i) * 1024);
    };

    // fragment read offsets inside a stage, per matrix-instruction k-step h
    int xoff[2], woff[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        xoff[h] = ((wm * WM + l16) * 8 + ((4 * h + lg) ^ chunk_swizzle<128>(l16))) * 16;
        woff[h] = XBYTES + (wn * WN + l16) * 64 + ((2 * h + (lg >> 1)) ^ ((l16 >> 2) & 3)) * 16 + (lg & 1) * 8;
    }

    const int n_lane = n0 + wn * WN + lg * 4;         // lane's channels: four per tile a
    const int soff = SOFF + (wn * WN + lg * 4) * 4;   // their scales inside a stage

    v4i acc[TN][TM];
    v4f facc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b) { acc[a][b] = v4i{0, 0, 0, 0}; facc[a][b] = v4f{0.f, 0.f, 0.f, 0.f}; }

    // prologue: k-tiles 0 .. NS-2
#pragma unroll
    for (int t = 0; t < NS - 1; ++t) issue(t < KT ? t : KT - 1, t);

    int st = 0;
    for (int kt = 0; kt < KT; ++kt) {
        wait_vmcnt<(NS - 2) * P>();                   // this wave's share of k-tile kt has landed
        __syncthreads();                              // ... everyone's; the stage of k-tile kt-1 is free
        const int nk = kt + NS - 1;
        issue(nk < KT ? nk : KT - 1, st == 0 ? NS - 1 : st - 1);

        const int8_t *stage = smem + st * STAGE;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            v4i af[TN], bf[TM];
#pragma unroll
            for (int a = 0; a < TN; ++a) {
                const uint2 p = *reinterpret_cast<const uint2 *>(stage + woff[h] + a * 16 * 64);
                af[a] = v4i{(int)((p.x << 4) & 0xF0F0F0F0u), (int)(p.x & 0xF0F0F0F0u),
                            (int)((p.y << 4) & 0xF0F0F0F0u), (int)(p.y & 0xF0F0F0F0u)};
            }
#pragma unroll
            for (int b = 0; b < TM; ++b) bf[b] = *reinterpret_cast<const v4i *>(stage + xoff[h] + b * 16 * BK);
            // the first half of a scale group starts from zero (a constant operand: no registers to clear)
#pragma unroll
            for (int a = 0; a < TN; ++a)
#pragma unroll
                for (int b = 0; b < TM; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[a], bf[b], h == 0 ? v4i{0, 0, 0, 0} : acc[a][b], 0, 0, 0);
        }

        // end of scale group kt: facc += s_w[kt][n] * (16 * sum)
#pragma unroll
        for (int a = 0; a < TN; ++a) {
            const float4 sca = *reinterpret_cast<const float4 *>(stage + soff + a * 64);
#pragma unroll
            for (int b = 0; b < TM; ++b) {
                if constexpr (DEBUG) {
                    const int64_t m = m0 + wm * WM + b * 16 + l16;
                    const int n = n_lane + a * 16;
                    if (m < g.M && n < g.N)
                        *reinterpret_cast<int4 *>(g.acc_debug + ((int64_t)kt * g.M + m) * g.N + n) =
                            make_int4(acc[a][b][0] >> 4, acc[a][b][1] >> 4, acc[a][b][2] >> 4, acc[a][b][3] >> 4);
                }
                facc[a][b][0] += sca.x * (float)acc[a][b][0];
                facc[a][b][1] += sca.y * (float)acc[a][b][1];
                facc[a][b][2] += sca.z * (float)acc[a][b][2];
                facc[a][b][3] += sca.w * (float)acc[a][b][3];
            }
        }
        st = (st + 1 == NS) ? 0 : st + 1;
    }
    wait_vmcnt<0>();                                  // the repeated copies of the last steps

    // epilogue: y = (s_x / 16) * facc + bias -> bf16
    const int64_t m_lane = m0 + wm * WM + l16;
    float sxm[TM], zcf[TM];
#pragma unroll
    for (int b = 0; b < TM; ++b) {
        const int64_t m = m_lane + b * 16;
        sxm[b] = m < g.M ? g.sx[m] * 0.0625f : 0.0f;
        zcf[b] = (ASYM && m < g.M) ? (float)g.zc[m] : 0.0f;
    }
    const bool full = m0 + BM <= g.M && n0 + BN <= g.N;      // workgroup-uniform
    constexpr int ROWB = WN * 2 + 16;
    if (full) __syncthreads();                        // the ring becomes the staging space below
    int8_t *const stg = smem + wave * (WM * ROWB);
    static_assert(4 * WM * (WN * 2 + 16) <= NS * STAGE, "staging space fits in the ring");
#pragma unroll
    for (int a = 0; a < TN; ++a) {
        const int n = n_lane + a * 16;
        const bool n_ok = n < g.N;
        float4 bi = make_float4(0.f, 0.f, 0.f, 0.f), cw = bi;
        if (g.bias && n_ok) bi = *reinterpret_cast<const float4 *>(g.bias + n);
        if (ASYM && n_ok) cw = *reinterpret_cast<const float4 *>(g.colsumw + n);
#pragma unroll
        for (int b = 0; b < TM; ++b) {
            const int64_t m = m_lane + b * 16;
            v4f t = facc[a][b];
            if constexpr (ASYM) t += v4f{zcf[b] * cw.x, zcf[b] * cw.y, zcf[b] * cw.z, zcf[b] * cw.w};
            uint2 o;
            o.x = pack_bf16x2(sxm[b] * t[0] + bi.x, sxm[b] * t[1] + bi.y);
            o.y = pack_bf16x2(sxm[b] * t[2] + bi.z, sxm[b] * t[3] + bi.w);
            if (full) *reinterpret_cast<uint2 *>(stg + (b * 16 + l16) * ROWB + (a * 16 + lg * 4) * 2) = o;
            else if (n_ok && m < g.M) *reinterpret_cast<uint2 *>(g.Y + m * g.ldy + n) = o;
        }
    }
    if (full) {
        // whole row segments, 16 bytes per lane (see epilogue_w8_rows)
        __builtin_amdgcn_wave_barrier();
        constexpr int LPR = WN / 8, RPI = 64 / LPR;
        const int r0 = lane / LPR, c = lane % LPR;
#pragma unroll
        for (int i = 0; i < WM / RPI; ++i) {
            const int row = i * RPI + r0;
            const uint4 v = *reinterpret_cast<const uint4 *>(stg + row * ROWB + c * 16);
            store_out16(g.Y + (m0 + wm * WM + row) * g.ldy + n0 + wn * WN + c * 8, v);
        }
    }
}

template <typename Kern>
hipError_t launch_kernel(Kern kern, const GemmArgs &a, int BM, int BN, size_t smem, hipStream_t st,
                         int threads = kThreads)
{
    GemmArgs g = a;
    g.tiles_m = (int)((g.M + BM - 1) / BM);
    g.tiles_n = (g.N + BN - 1) / BN;
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), smem); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(g.tiles_m * g.tiles_n)), dim3(threads), smem, st, g);
    return hipGetLastError();
}

template <int BM, int BN, int NS, int WGM, int WGN>
hipError_t launch_ring4(const GemmArgs &a, bool debug, hipStream_t st)
{
    const size_t smem = (size_t)NS * (BM * 128 + BN * 64 + 1024);
    if (a.zc) {
        if (!a.colsumw) return hipErrorInvalidValue;
        if (debug) return launch_kernel(qgemm4_ring_kernel<BM, BN, NS, WGM, WGN, true, true>, a, BM, BN, smem, st);
        return launch_kernel(qgemm4_ring_kernel<BM, BN, NS, WGM, WGN, false, true>, a, BM, BN, smem, st);
    }
    if (debug) return launch_kernel(qgemm4_ring_kernel<BM, BN, NS, WGM, WGN, true>, a, BM, BN, smem, st);
    return launch_kernel(qgemm4_ring_kernel<BM, BN, NS, WGM, WGN, false>, a, BM, BN, smem, st);
}

// the kernel that takes every shape with asymmetric activations (ring, 128 x 128 x 64, four stages)
hipError_t launch_ring_asym(const GemmArgs &a, bool debug, hipStream_t st)
{
    constexpr int BM = 128, BN = 128, BK = 64, NS = 4;
    const size_t smem = (size_t)NS * (BM + BN) * BK;
    if (debug) return launch_kernel(qgemm8_ring_kernel<BM, BN, BK, NS, 2, 2, true, true>, a, BM, BN, smem, st);
    return launch_kernel(qgemm8_ring_kernel<BM, BN, BK, NS, 2, 2, false, true>, a, BM, BN, smem, st);
}

template <int BM, int BN, int BK, int NS, int WGM, int WGN>
hipError_t launch_ring(const GemmArgs &a, bool debug, hipStream_t st)
{
    if (a.zc) return launch_ring_asym(a, debug, st);
    const size_t smem = (size_t)NS * (BM + BN) * BK;
    if (debug) return launch_kernel(qgemm8_ring_kernel<BM, BN, BK, NS, WGM, WGN, true>, a, BM, BN, smem, st);
    return launch_kernel(qgemm8_ring_kernel<BM, BN, BK, NS, WGM, WGN, false>, a, BM, BN, smem, st);
}

template <int BM, int BN, int NS, int WGM, int WGN>
hipError_t launch_pipe(const GemmArgs &a, bool debug, hipStream_t st)
{
    // the pipelined kernel takes full tiles only; ragged shapes go to the ring kernel
    if (a.M % BM != 0 || a.N % BN != 0) return launch_ring<128, 128, 64, 4, 2, 2>(a, debug, st);
    constexpr int NW = WGM * WGN;
    const size_t smem = (size_t)NS * (BM * 128 + NW * ((BN / 8 + NW - 1) / NW) * 1024);
    if (a.zc) {
        // asymmetric activations: built for the 128 x 144 tiles only; a block of LDS per wave for the zero-point operands
        if constexpr (BM == 128 && BN == 144 && NW == 4) {
            const size_t smem_z = smem + NW * kZpBlock;
            if (debug) return launch_kernel(qgemm8_pipe_kernel<BM, BN, NS, WGM, WGN, true, true>, a, BM, BN, smem_z, st, NW * 64);
            return launch_kernel(qgemm8_pipe_kernel<BM, BN, NS, WGM, WGN, false, true>, a, BM, BN, smem_z, st, NW * 64);
        } else {
            return launch_ring_asym(a, debug, st);
        }
    }
    if (debug) return launch_kernel(qgemm8_pipe_kernel<BM, BN, NS, WGM, WGN, true>, a, BM, BN, smem, st, NW * 64);
    return launch_kernel(qgemm8_pipe_kernel<BM, BN, NS, WGM, WGN, false>, a, BM, BN, smem, st, NW * 64);
}

template <int BM, int BN, int NS, int WGM, int WGN>
hipError_t launch_pipe2(const GemmArgs &a, bool debug, hipStream_t st)
{
    // full tiles and at least NS k-tiles per wave group; else the one-group kernel
    if (a.M % BM != 0 || a.N % BN != 0 || a.K / 256 < NS) return launch_pipe<BM, BN, 2 * NS, WGM, WGN>(a, debug, st);
    const size_t smem = (size_t)2 * NS * (BM * 128 + 4 * ((BN / 8 + 3) / 4) * 1024) + (a.zc ? 8 * kZpBlock : 0);
    GemmArgs g = a;
    g.tiles_m = (int)(g.M / BM);
    g.tiles_n = g.N / BN;
    auto go = [&](auto kern) -> hipError_t {
        if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), smem); e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3((unsigned)(g.tiles_m * g.tiles_n)), dim3(2 * kThreads), smem, st, g);
        return hipGetLastError();
    };
    if (a.zc) {
        if (debug) return go(qgemm8_pipe2_kernel<BM, BN, NS, WGM, WGN, true, true>);
        return go(qgemm8_pipe2_kernel<BM, BN, NS, WGM, WGN, false, true>);
    }
    if (debug) return go(qgemm8_pipe2_kernel<BM, BN, NS, WGM, WGN, true>);
    return go(qgemm8_pipe2_kernel<BM, BN, NS, WGM, WGN, false>);
}

template <int BM, int BN, int NS, int WGM, int WGN, int WGS_PER_CU>
hipError_t launch_persist(const GemmArgs &a, bool debug, hipStream_t st)
{
    // full tiles and at least NS k-tiles; everything else goes to the ring kernel
    if (a.M % BM != 0 || a.N % BN != 0 || a.K / 128 < NS) return launch_ring<128, 128, 64, 4, 2, 2>(a, debug, st);
    GemmArgs g = a;
    g.tiles_m = (int)(g.M / BM);
    g.tiles_n = g.N / BN;
    const size_t smem = (size_t)NS * (BM + BN) * 128;
    auto kern = debug ? qgemm8_persist_kernel<BM, BN, NS, WGM, WGN, true>
                      : qgemm8_persist_kernel<BM, BN, NS, WGM, WGN, false>;
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), smem); e != hipSuccess) return e;
    int grid = num_cus() * WGS_PER_CU;
    if (grid > g.tiles_m * g.tiles_n) grid = g.tiles_m * g.tiles_n;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kThreads), smem, st, g);
    return hipGetLastError();
}

}  // namespace

// int4 weights: 0: 128x128 NS3 (two workgroups per compute unit)   1: 128x128 NS2 (three)
// asymmetric activations (a.zc, a.colsum set).  kind: 0 ring (any shape); 14, 15, 18: the 128 x 144
// kernels of the table below (they fall back to the ring kernel for shapes they do not take)
hipError_t launch_qgemm8_asym(const GemmArgs &a, bool debug, int kind, hipStream_t st)
{
    if ((!a.zc && !a.zcw) || !a.colsum || a.K % 128 != 0 || a.N < 4) return hipErrorInvalidValue;
    if (a.zcw && !a.rowsum) return hipErrorInvalidValue;
    // the pipelined kernels multiply column sums as 24-bit values and carry the activations' term only:
    // long K and asymmetric weights take the kernel that adds the terms in its epilogue
    if (a.K >= 65536 || a.zcw) kind = 0;
    switch (kind) {
        case 0: return launch_ring_asym(a, debug, st);
        case 14: return launch_pipe<128, 144, 4, 4, 1>(a, debug, st);
        case 15: return launch_pipe<128, 144, 2, 4, 1>(a, debug, st);
        case 18: return launch_pipe2<128, 144, 2, 4, 1>(a, debug, st);
    }
    return hipErrorInvalidValue;
}

int dma4_num_variants() { return 2; }

hipError_t launch_qgemm4_dma(const GemmArgs &a, bool debug, int variant, hipStream_t st)
{
    if (a.K % 128 != 0 || a.N < 4) return hipErrorInvalidValue;
    switch (variant) {
        case 0: return launch_ring4<128, 128, 3, 2, 2>(a, debug, st);
        case 1: return launch_ring4<128, 128, 2, 2, 2>(a, debug, st);
    }
    return hipErrorInvalidValue;
}

// ring: 0: 128x128x64 NS4   1: 256x128x64 NS4   2: 128x256x64 NS4   3: 128x128x128 NS3   4: 256x128x128 NS3
// pipe: 5: 256x128 NS3   6: 128x128 NS4   7: 128x256 NS3   8: 256x256 NS2   9: 128x128 NS2
// persistent: 10: 128x128 NS2 (2 workgroups per CU)   11: 256x128 NS3   12: 128x256 NS3   13: 128x128 NS4
// pipe, 144-channel tiles (1152 = 8 x 144: the DiT-XL/2 widths give whole rounds of 256 tiles): 14: 128x144 NS4   15: 128x144 NS2 (two workgroups per CU)
// 256 tokens x 144 channels (waves 64 x 144): 16: NS2   17: NS3
// 18: 128x144, two wave groups splitting K inside the workgroup, two stages each
// 19: 256x144 NS2 with eight waves (32 x 144 each): two 128-token halves sharing one copy of the weight tile
int dma_num_variants() { return 20; }

hipError_t launch_qgemm8_dma(const GemmArgs &a, bool debug, int variant, hipStream_t st)
{
    switch (variant) {
        case 0: return launch_ring<128, 128, 64, 4, 2, 2>(a, debug, st);
        case 1: return launch_ring<256, 128, 64, 4, 2, 2>(a, debug, st);
        case 2: return launch_ring<128, 256, 64, 4, 2, 2>(a, debug, st);
        case 3: return launch_ring<128, 128, 128, 3, 2, 2>(a, debug, st);
        case 4: return launch_ring<256, 128, 128, 3, 2, 2>(a, debug, st);
        case 5: return launch_pipe<256, 128, 3, 2, 2>(a, debug, st);
        case 6: return launch_pipe<128, 128, 4, 2, 2>(a, debug, st);
        case 7: return launch_pipe<128, 256, 3, 2, 2>(a, debug, st);
        case 8: return launch_pipe<256, 256, 2, 2, 2>(a, debug, st);
        case 9: return launch_pipe<128, 128, 2, 2, 2>(a, debug, st);
        case 10: return launch_persist<128, 128, 2, 2, 2, 2>(a, debug, st);
        case 11: return launch_persist<256, 128, 3, 2, 2, 1>(a, debug, st);
        case 12: return launch_persist<128, 256, 3, 2, 2, 1>(a, debug, st);
        case 13: return launch_persist<128, 128, 4, 2, 2, 1>(a, debug, st);
        case 14: return launch_pipe<128, 144, 4, 4, 1>(a, debug, st);
        case 15: return launch_pipe<128, 144, 2, 4, 1>(a, debug, st);
        case 16: return launch_pipe<256, 144, 2, 4, 1>(a, debug, st);
        case 17: return launch_pipe<256, 144, 3, 4, 1>(a, debug, st);
        case 18: return launch_pipe2<128, 144, 2, 4, 1>(a, debug, st);
        case 19: return launch_pipe<256, 144, 2, 8, 1>(a, debug, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace gemm
}  // namespace trdq
