// Internal declarations shared by the host API and the HIP kernels of libtrdq.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "trdq.h"

namespace trdq {

constexpr int kBlock = TRDQ_BLOCK;  // rotation block = int4 scale group

// The transform folded into a weight set; the fused kernel and the layer object apply kRotHadamard only.
enum { kRotHadamard = 0, kRotHadamardRPR = 1, kRotDense = 2, kRotDenseRPR = 3 };

// Device-side weight set of one time-step group (H_t(W) of Eq. 10, quantised).
//   wbits 8: codes = int8  [N, K]   (K contiguous: the transposed canonical matrix)
//   wbits 4: codes = uint8 [N, K/2]; every 4 bytes hold 8 consecutive k of one output
//            channel: byte j = code(k0+j) & 0xF | (code(k0+4+j) & 0xF) << 4, so that
//            (v << 4) & 0xF0F0F0F0 and v & 0xF0F0F0F0 give 16*code as packed int8.
//   scales : float32 [N] (wbits 8) or [K/128, N] (wbits 4), the true s_w.
struct Weights {
    int K = 0, N = 0;
    int wbits = 0;               // storage layout: 8 (one code per byte) or 4 (packed nibbles, group scales)
    int qbits = 0;               // width of the codes: 8, 6 (in the 8-bit layout) or 4
    void *codes = nullptr;
    float *scales = nullptr;
    void *codes_tiled = nullptr; // int8 weights with N % 144 == 0: the same codes in 1 KB blocks of 16 channels x 64 k
    int rotation = 0;            // which transform was folded in (kRot*): the activation side must apply the same one
    int32_t *colsum = nullptr;   // int8 weights: sum over k of the codes of every output channel [N]
    int32_t *zcw = nullptr;      // asymmetric int8 weights (Eq. 1-3 per output channel): 128 - z_w [N]; codes hold q - 128
    float *colsumw = nullptr;    // int4 weights: 16 * sum_g s_w[g][n] * (sum of the codes of group g) [N]
    int device = 0;
};

// Dense rotation blocks (the BlockDiag equation with arbitrary orthogonal blocks, e.g. Eq. 6-7):
// the float32 blocks and the diagonal for the weight side, and the blocks with the diagonal folded
// in, split into bf16 pieces in matrix-instruction fragment order, for the activation side.
struct Rotation {
    int K = 0;
    float *R = nullptr;          // [K/128][128][128]
    float *diag = nullptr;       // [K] or null (ones)
    void *pieces = nullptr;      // diag . R_b as bf16 pieces (operand of a first or only rotation)
    void *frags32 = nullptr;     // R_b as float fragments (operand of a second rotation)
    int device = 0;
};

struct Table {
    int n_steps = 0, n_groups = 0;
    int32_t *map = nullptr;
};

// Kernel launchers (defined in the .hip files).  All return hipError_t of the launch.
// warm / warm_bytes: optional device range (16-byte aligned, a multiple of 16 bytes) that the
// kernel reads once and discards, to pull it into the memory-side cache for the next kernel.
// zc: null (symmetric quantiser), or where the asymmetric quantiser writes 128 - z_i per token.
// tiled: Xq is written in 1 KB blocks of 16 tokens x 64 k (block (m / 16, k / 64) at ((m / 16) * K / 64 + k / 64) * 1024)
hipError_t launch_rotate_quant(const uint16_t *X, int64_t M, int K, int64_t ldx, const float *diag,
                               int8_t *Xq, float *sx, int32_t *zc, const void *warm, int64_t warm_bytes, hipStream_t st,
                               int abits = 8,    // symmetric codes in +-(2^(abits-1) - 1); K <= 4608 unless 8
                               bool tiled = false);
// the product on block-tiled operands, and the conversion between the two forms of an int8 matrix [R, K]
bool qgemm_tiled_supports(const Weights &w, int64_t M, const void *Y, int64_t ldy);
hipError_t launch_qgemm_tiled(const Weights &w, const int8_t *Xt, const float *sx, int64_t M, const float *bias,
                              uint16_t *Y, int64_t ldy, int32_t *acc_debug, hipStream_t st);
// measured choice between the two products for a layer object (true: the tiled pair is the faster one)
bool qgemm_tiled_pays(int64_t M, int K, int N);
hipError_t launch_retile_rows(const int8_t *src, int8_t *dst, int64_t R, int K, bool to_tiled, hipStream_t st);
hipError_t launch_retile_w4_codes(const void *src, void *dst, int64_t N, int K, hipStream_t st);
hipError_t launch_rotate_quant_wide(const uint16_t *X, int64_t M, int K, int64_t ldx, const float *diag,
                                    int8_t *Xq, float *sx, hipStream_t st);

// Full transform of Eq. 9 (rotation, permutation, rotation) and per-token quantisation.
bool rotate_quant_rpr_supports(int K);
hipError_t launch_rotate_quant_rpr(const uint16_t *X, int64_t M, int K, int64_t ldx, const float *diag,
                                   const int32_t *perm, int8_t *Xq, float *sx, const void *warm, int64_t warm_bytes,
                                   hipStream_t st, int32_t *zc = nullptr);   // zc: asymmetric codes, as launch_rotate_quant

// perm (optional): rows are read through it (row k of the input to the rotation = row perm[k]).
// norm: what undoes the unnormalised butterflies (1/sqrt(128) per rotation applied).
hipError_t launch_prepare_rotate(const float *W, int K, int N, const float *diag, const int32_t *perm,
                                 float *Wrot, float *amax, hipStream_t st);
// asymmetric weight quantiser: lohi = scratch of 2 N floats; codes [N, K] = q - 128, scales [N], zcw [N] = 128 - z
hipError_t launch_prepare_quant_asym(const float *Wrot, float *lohi, int K, int N, float norm, void *codes, float *scales,
                                     int32_t *zcw, hipStream_t st);
hipError_t launch_xq_rowsum(const int8_t *Xq, int64_t M, int K, int32_t *rowsum, hipStream_t st);
hipError_t launch_weight_colsumw4(const void *codes, const float *scales, int K, int N, float *colsumw, hipStream_t st);
hipError_t launch_prepare_quant(const float *Wrot, const float *amax, int K, int N, int wbits, float norm,
                                void *codes, float *scales, hipStream_t st);   // wbits 8, 6 (8-bit layout) or 4

// Calibration-side reductions (calibrate.hip).  mag / wmax / d are device arrays of K floats.
hipError_t launch_channel_absmax(const uint16_t *X, int64_t M, int K, int64_t ldx, const float *diag,
                                 bool rotate, float *mag, hipStream_t st);
hipError_t launch_weight_row_absmax(const float *W, int K, int N, float *wmax, hipStream_t st);
hipError_t launch_smooth_diag(const float *xmax, const float *wmax, int K, float alpha, float *d, hipStream_t st);

int qgemm_num_variants();
// colsum[n] = sum_k codes[n][k] for int8 codes stored [N][K]
hipError_t launch_weight_colsum(const void *codes, int K, int N, int32_t *colsum, hipStream_t st);
// zc: null, or the per-token zero-point terms of asymmetric activations (int8 weights only)
// rowsum: with asymmetric weights (w.zcw), the per-token sums of the activation codes as stored
hipError_t launch_qgemm(const Weights &w, const int8_t *Xq, const float *sx, const int32_t *zc, int64_t M,
                        const float *bias, uint16_t *Y, int64_t ldy, int32_t *acc_debug,
                        int variant, hipStream_t st, const int32_t *rowsum = nullptr);

hipError_t launch_cosine_similarity(const uint16_t *A, const uint16_t *B, int n_seg, int64_t seg_len,
                                    int64_t stride_a, int64_t stride_b, double *acc_ws, float *out, hipStream_t st);
// Most segments the entry point without a workspace argument takes, and the current device's address of its
// file-scope accumulator array (looked up once per device, with that device current; thread-safe).
constexpr int kCosineStaticMaxSeg = TRDQ_COSINE_STATIC_MAX_SEG;
hipError_t cosine_static_scratch(double **out);
// Raises a kernel's dynamic-LDS limit to at least `bytes` on the current device.  The attribute
// belongs to the (kernel, device) pair; what has been set is remembered per pair, so the HIP call
// happens once for each and callers may ask before every launch (thread-safe).
hipError_t ensure_dynamic_lds(const void *kernel, size_t bytes);
// Compute units of the current device (read once per device; 256 if the query fails).
int num_cus();

// yardstick kernels (peaks.hip)
int peak_mfma_independent();
hipError_t launch_peak_mfma_i8(int32_t *sink, int workgroups, int waves, int iters, hipStream_t st, bool random_data = false);
hipError_t launch_peak_stream(const void *src, void *dst, int64_t n_elems, hipStream_t st);
size_t greedy_workspace_bytes(int64_t Mc, int K);
hipError_t launch_greedy_rotation(const uint16_t *X, int64_t Mc, int K, int64_t ldx, const float *diag,
                                  const float *R1, const int32_t *perm,   // null, or: start from ((X d) R1)[:, perm]
                                  const double *Q, int n_steps, void *workspace, float *R_out, int *n_out_dev,
                                  hipStream_t st);
hipError_t launch_channel_absmax_dense(const uint16_t *X, int64_t M, int K, int64_t ldx, const void *pieces,
                                       float *mag, hipStream_t st);
size_t rotation_pieces_bytes(int K);
hipError_t launch_rotation_pieces(const float *R, const float *diag, int K, void *pieces, hipStream_t st);
bool rotate_quant_dense_supports(int K);
hipError_t launch_rotate_quant_dense(const uint16_t *X, int64_t M, int K, int64_t ldx, const void *pieces,
                                     int8_t *Xq, float *sx, hipStream_t st);
hipError_t launch_prepare_rotate_dense(const float *W, int K, int N, const float *diag, const int32_t *perm,
                                       const float *R, float *Wrot, float *amax, hipStream_t st);
size_t rotation_frags32_bytes(int K);
hipError_t launch_rotation_frags32(const float *R, int K, void *frags, hipStream_t st);
bool rotate_quant_dense_rpr_supports(int K);
hipError_t launch_rotate_quant_dense_rpr(const uint16_t *X, int64_t M, int K, int64_t ldx, const void *pieces1,
                                         const int32_t *perm, const void *frags2, int8_t *Xq, float *sx, hipStream_t st);
// wide rows (more than 12 blocks) through a workspace of once-rotated values; pieces2: the second rotation's bf16 pieces
size_t rotate_quant_dense_rpr_workspace_bytes(int64_t M, int K);
hipError_t launch_rotate_quant_dense_rpr_ws(const uint16_t *X, int64_t M, int K, int64_t ldx, const void *pieces1,
                                            const int32_t *perm, const void *pieces2, int8_t *Xq, float *sx,
                                            float *T, hipStream_t st);
bool fused_supports(int K);
bool fused_pays(int64_t M, int K, int N, int wbits);
hipError_t launch_linear_fused(const Weights &w, const uint16_t *X, int64_t M, int64_t ldx,
                               const float *diag, const float *bias, uint16_t *Y, int64_t ldy,
                               hipStream_t st, bool asym = false);

}  // namespace trdq
