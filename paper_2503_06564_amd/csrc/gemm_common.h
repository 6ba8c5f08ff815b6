// Shared pieces of the integer-product kernels: argument block, tile -> die mapping.
#pragma once

#include "device_utils.h"
#include "trdq_internal.h"

namespace trdq {
namespace gemm {

constexpr int kThreads = 256;

struct GemmArgs {
    const int8_t *Xq;      // [M, K]
    const void *Wc;        // codes, see Weights
    const float *sx;       // [M]
    const float *sw;       // [N] or [K/128, N]
    const float *bias;     // [N] or null
    uint16_t *Y;           // [M, ldy]
    int32_t *acc_debug;    // null, [M, N] or [K/128, M, N]
    // asymmetric activations: zc[i] = 128 - z_i per token, and with int8 weights the column sums of the
    // weight codes (the integer sum of a product is acc + zc[i] * colsum[n]), with int4 weights
    // colsumw[n] = 16 * sum_g s_w[g][n] * colsum_g[n] (the scaled term, added in float).  Null otherwise.
    const int32_t *zc = nullptr;
    const int32_t *colsum = nullptr;
    const float *colsumw = nullptr;
    // asymmetric weights: zcw[n] = 128 - z_w[n] and rowsum[i] = sum_k Xq[i][k] of the stored activation codes; the
    // integer sum of the product is acc + zc[i] colsum[n] + zcw[n] (rowsum[i] + K zc[i]).  Null otherwise.
    const int32_t *zcw = nullptr;
    const int32_t *rowsum = nullptr;
    int64_t M, ldy;
    int K, N;
    int tiles_m, tiles_n;
};

// Workgroups are handed to the 8 accelerator dies (XCDs) round-robin by their linear id; give
// each die a contiguous run of tiles so that the panels it re-reads stay in its own L2.
__device__ __forceinline__ int xcd_remap(int bid, int ntiles)
{
    const int q = ntiles >> 3, r = ntiles & 7;
    const int xcd = bid & 7, idx = bid >> 3;
    return xcd * q + (xcd < r ? xcd : r) + idx;
}

// Work item id -> tile coordinates.  Each die owns a band of token panels; inside the band the
// tiles are visited in groups of up to 8 token panels, channel tile by channel tile, so the
// ~64 tiles a die has in flight form an 8 x 8 block: 8 activation panels + 8 weight panels fit
// its 4 MB L2, instead of every round streaming the whole weight matrix through it.
// (Needs tiles_m % 8 == 0; otherwise the plain run-per-die order is used.)
// Every die pulls what it touches through its own L2: with 8 bands that is the activations once
// and the weights 8 times.  When the weights are the larger part of that (few token panels, many
// channel tiles) the dies form a 4 x 2 grid instead -- 4 bands, each split between two dies by
// channel halves -- which fetches the activations twice and the weights 4 times.
__device__ __forceinline__ void tile_map(int id, int tiles_m, int tiles_n, int &tm, int &tn)
{
    if ((tiles_m & 7) == 0) {
        const int xcd = id & 7, i = id >> 3;         // i-th work item of this die
        const bool halves = (tiles_n & 1) == 0 && 8 * tiles_n > 3 * tiles_m;
        const int per = halves ? tiles_m >> 2 : tiles_m >> 3;     // token panels per die
        const int cols = halves ? tiles_n >> 1 : tiles_n;          // channel tiles per die
        const int gm = per < 8 ? per : 8;
        const int group = i / (gm * cols);
        const int j = i - group * gm * cols;
        const int rows = (per - group * gm) < gm ? (per - group * gm) : gm;   // last group may be short
        const int c = j / rows;
        tn = (halves ? (xcd >> 2) * cols : 0) + c;
        tm = (halves ? (xcd & 3) : xcd) * per + group * gm + (j - c * rows);
    } else {
        const int t = xcd_remap(id, tiles_m * tiles_n);
        tm = t / tiles_n;
        tn = t - tm * tiles_n;
    }
}

// ---- pieces shared by the direct-to-LDS kernels ---------------------------------------------------

// row -> XOR mask of the 16-byte chunk index, a function of (row mod 16) only so that the
// fragment offsets of different 16-row tiles differ by a constant.
//
// The LDS has 64 four-byte banks (256 B per clock).  A 128-bit read of a wavefront is served
// 16 lanes per clock, and (measured by swapping lane addresses in a conflict-free pattern) the
// lanes served together are the four-lane quads {0,3,5,6}, {1,2,4,7}, {9,10,12,15} and
// {8,11,13,14}.  With the matrix-instruction operand layout (lane = row + 16 * chunk) each of
// those sets holds every row once, rows 0-3 and 12-15 with one chunk of a pair and rows 4-11
// with the other.  The masks below send the 16 lanes of every set to 16 different 16-byte
// bank groups, for row strides of 64 B and 128 B.
template <int BK>
__device__ __forceinline__ int chunk_swizzle(int row)
{
    const int r = row & 15;
    if constexpr (BK == 64) return (r >> 3) << 1;
    else return (r & 2) | ((r >> 1) & 4);
}

__device__ __forceinline__ void dma_1k(uint32_t voff, const void *sbase, uint32_t lds_addr)
{
    // one wait state between the scalar write of M0 and the copy that reads it
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(sbase), "s"(lds_addr) : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// Direct-to-LDS int8 kernels (qgemm_dma.hip).  variant indexes the table in that file.
int dma_num_variants();
hipError_t launch_qgemm8_dma(const GemmArgs &a, bool debug, int variant, hipStream_t st);
// the kernel for asymmetric activations (a.zc and a.colsum set): 128 x 128 ring kernel, any shape
hipError_t launch_qgemm8_asym(const GemmArgs &a, bool debug, int kind, hipStream_t st);

// int4-weight kernels on the same path (qgemm_dma.hip).
int dma4_num_variants();
hipError_t launch_qgemm4_dma(const GemmArgs &a, bool debug, int variant, hipStream_t st);

// Kernel on block-tiled operands (qgemm_tiled.hip): a.Xq and a.Wc point at the tiled forms.
bool tiled_supports(const GemmArgs &a);
hipError_t launch_qgemm8_tiled(const GemmArgs &a, bool debug, hipStream_t st);
hipError_t launch_retile(const int8_t *src, int8_t *dst, int64_t R, int K, bool to_tiled, hipStream_t st);
// int4 weights on block-tiled operands (qgemm_tiled.hip): a.Wc holds the block form of the packed codes
bool tiled4_supports(const GemmArgs &a);
hipError_t launch_qgemm4_tiled(const GemmArgs &a, bool debug, hipStream_t st);
hipError_t launch_retile_w4(const void *src, void *dst, int64_t N, int K, hipStream_t st);

// 256 x 256 tile kernel with a hand-scheduled main loop (qgemm_wide.hip).
bool wide_supports(const GemmArgs &a);
hipError_t launch_qgemm8_wide(const GemmArgs &a, bool debug, hipStream_t st);

}  // namespace gemm
}  // namespace trdq
