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
    int64_t M, ldy;
    int K, N;
    int tiles_m, tiles_n;
};

// Workgroups are handed to the 8 accelerator dies round-robin by their linear id; give each
// die a contiguous run of tiles (a few token panels times all channel tiles) so that the
// panels it re-reads stay in its own L2.
__device__ __forceinline__ int xcd_remap(int bid, int ntiles)
{
    const int q = ntiles >> 3, r = ntiles & 7;
    const int xcd = bid & 7, idx = bid >> 3;
    return xcd * q + (xcd < r ? xcd : r) + idx;
}


// Direct-to-LDS int8 kernels (qgemm_dma.hip).  variant indexes the table in that file.
int dma_num_variants();
hipError_t launch_qgemm8_dma(const GemmArgs &a, bool debug, int variant, hipStream_t st);

}  // namespace gemm
}  // namespace trdq
