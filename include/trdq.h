/*
 * trdq.h -- C ABI of libtrdq: the rotated W8A8 / W4A8 linear layer of TR-DQ
 * (Time-Rotation Diffusion Quantization) on AMD MI355X (gfx950).
 *
 * The layer computes, for the linear Y = X . W of a denoiser at sampling
 * step t (paper Sec. 3.1, Eq. 10):
 *
 *     F_t(X_t, W) = G_t(X_t) . H_t(W)
 *     G_t(X) = (X . Delta_t) . R            (online, per call)
 *     H_t(W) = R^T . (Delta_t^-1 . W)       (offline, once per time-step group)
 *
 * with R block-diagonal, each 128 x 128 block the orthonormal Sylvester
 * Hadamard matrix (the BlockDiag equation of Sec. 3.2 with 2^n = 128; the
 * permutation P and the second rotation of Eq. 9 are the identity here).
 * G_t(X) is quantised per token to int8 with a scale computed online from the
 * row's largest magnitude; H_t(W) is quantised per output channel to int8 or
 * per (128-input-channel group, output channel) to int4 (Eq. 1-2 in their
 * symmetric form: scale = absmax / (2^(b-1) - 1), no zero point, nearest
 * rounding, ties to even).  The product runs on the int8 matrix cores with
 * int32 accumulation and is rescaled (and biased) to bf16 in the epilogue.
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses on the current HIP device,
 *     "host" pointers are ordinary host memory.  The caller owns every buffer
 *     it passes; the library owns the objects it returns through `** out`
 *     until the matching *_destroy call.
 *   - Matrices are row-major.  X is [M, K] (tokens x C_in), W is [K, N]
 *     (C_in x C_out, as in the paper -- the transpose of a torch Linear
 *     weight), Y is [M, N].  bf16 values are passed as 16-bit patterns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Online calls (rotate_quant, qgemm, linear_fused, layer_forward) are
 *     asynchronous on that stream and allocate nothing.  prepare_weights
 *     allocates device memory; the export calls synchronise.
 *   - Every call returns a trdq_status.  All argument checks happen before
 *     the first HIP call, so they can be exercised on a machine with no GPU.
 *     Nothing is printed and nothing aborts.  M == 0 is a valid no-op, for which the
 *     data pointers may be NULL (an empty tensor has no storage).
 *   - NaN / Inf in X or W are not detected; the result is then unspecified.
 *   - Handles are immutable after creation: concurrent forward calls on
 *     different streams may share them.  A handle's buffers live on the device
 *     that was current when it was created; a launch that is given a handle
 *     while another device is current returns ERR_MISMATCH.
 */
#ifndef TRDQ_H
#define TRDQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum trdq_status {
    TRDQ_OK = 0,
    TRDQ_ERR_NULL = 1,        /* a required pointer is NULL */
    TRDQ_ERR_SHAPE = 2,       /* K % 128 != 0, K/N <= 0, M < 0, leading dimension too small, misaligned pointer */
    TRDQ_ERR_RANGE = 3,       /* step or group out of range, bad table */
    TRDQ_ERR_UNSUPPORTED = 4, /* wbits not in {4, 6, 8}, block != 128, shape beyond a kernel's limit */
    TRDQ_ERR_MISMATCH = 5,    /* handle's K / N / width does not match the call */
    TRDQ_ERR_ALLOC = 6,       /* host or device allocation failed */
    TRDQ_ERR_HIP = 7          /* a HIP runtime call or kernel launch failed */
} trdq_status;

#define TRDQ_BLOCK 128        /* rotation block = int4 scale group, in input channels */

const char *trdq_status_str(trdq_status s);

/* Version of the ABI declared in this header (major * 100 + minor). */
int trdq_abi_version(void);

/* ------------------------------------------------------------------ table
 * Time-step -> group table: the diagonal, rotation and permutation in use depend on
 * the sampling step (Sec. 3.2, the paragraph on time-step awareness; t in {1..N},
 * Eq. 10; indexed here by sampling-step index 0..n_steps-1).  Host object. */
typedef struct trdq_table trdq_table;

/* map_host: n_steps entries in [0, n_groups), copied; NULL selects the contiguous
 * near-equal partition g = floor(step * n_groups / n_steps).
 * Errors: NULL out -> ERR_NULL; n_steps <= 0, n_groups <= 0, n_groups > n_steps
 * or a map entry outside [0, n_groups) -> ERR_RANGE. */
trdq_status trdq_table_create(int n_steps, int n_groups, const int32_t *map_host, trdq_table **out);
trdq_status trdq_table_lookup(const trdq_table *t, int step, int *group_out);
trdq_status trdq_table_sizes(const trdq_table *t, int *n_steps_out, int *n_groups_out);
void trdq_table_destroy(trdq_table *t);

/* ---------------------------------------------------------------- weights
 * Offline weight transform and quantisation, H_t(W) of Eq. 10 followed by the
 * per-channel weight quantiser (Sec. 3.1).  One handle per time-step group. */
typedef struct trdq_weights trdq_weights;

/* W_dev:    float32 [K, N] row-major, device.  Not modified, not retained.
 * diag_dev: float32 [K], device: this group's Delta (activations are multiplied
 *           by it, weight rows divided); NULL = all ones.  Entries must be non-zero.
 * block:    must be 128.   wbits: 8 (scale per output channel, codes in [-127,127])
 *           or 4 (scale per 128-row group and output channel, codes in [-7,7]).
 * The call enqueues its kernels on `stream` and synchronises it before returning
 * (temporary buffers are freed).  *out holds codes and scales in a private,
 * matrix-core friendly layout.
 * Errors: NULL W_dev/out -> ERR_NULL; K <= 0, N <= 0, K % 128 != 0, N % 16 != 0
 * -> ERR_SHAPE; block != 128 or wbits not 4/6/8 -> ERR_UNSUPPORTED
 * (wbits 6: see "other bit-widths" below). */
trdq_status trdq_prepare_weights(const float *W_dev, int K, int N, const float *diag_dev,
                                 int block, int wbits, void *stream, trdq_weights **out);

trdq_status trdq_weights_info(const trdq_weights *w, int *K_out, int *N_out, int *wbits_out);

/* Canonical copies on the host (synchronises the device):
 * codes_host  int8 [K, N], one code per byte for both widths (may be NULL);
 * scales_host float32, [N] for wbits 8, [K/128, N] for wbits 4 (may be NULL). */
trdq_status trdq_weights_export(const trdq_weights *w, int8_t *codes_host, float *scales_host);

/* wbits 4 only: packed_host uint8 [K/2, N], byte (j, n) = code(2j, n) & 0xF | (code(2j+1, n) & 0xF) << 4
 * (two's complement nibbles, even k in the low nibble).  wbits 8 -> ERR_MISMATCH. */
trdq_status trdq_weights_export_packed(const trdq_weights *w, uint8_t *packed_host);

/* Bytes of the weight format (codes + scales): K*N + 4N for wbits 8, K*N/2 + 4*(K/128)*N for wbits 4.
 * An int8 set whose N is a multiple of 144, and an int4 set whose N is a multiple of 128, holds
 * its codes a second time, block-tiled for trdq_qgemm_tiled (another K*N resp. K*N/2 bytes of
 * device memory, not part of this figure). */
trdq_status trdq_weights_nbytes(const trdq_weights *w, int64_t *nbytes_out);

void trdq_weights_destroy(trdq_weights *w);

/* ----------------------------------------------------------------- online
 * G_t(X_t) of Eq. 10 followed by the per-token dynamic quantiser (Sec. 3.1,
 * Eq. 1-2 symmetric; the scale comes from the row itself at run time, Sec. 3.2):
 *   V = (X . diag) . R,   s_x[i] = max_k |V[i,k]| / 127,
 *   Xq[i,k] = rint(V[i,k] / s_x[i]);   an all-zero row gives s_x = 0, codes 0.
 * X_dev:  bf16 [M, K], row stride ldx elements (ldx >= K, ldx % 8 == 0, 16-byte aligned base).
 * Xq_dev: int8 [M, K] dense (16-byte aligned).   sx_dev: float32 [M].
 * Errors: NULL X/Xq/sx -> ERR_NULL; M < 0, K <= 0, K % 128, ldx < K, misalignment
 * -> ERR_SHAPE; block != 128 -> ERR_UNSUPPORTED. */
trdq_status trdq_rotate_quant(const void *X_dev, int64_t M, int K, int64_t ldx,
                              const float *diag_dev, int block,
                              int8_t *Xq_dev, float *sx_dev, void *stream);

/* The same pass, which additionally reads the codes of `next` (the weights of the product that
 * follows; NULL = plain trdq_rotate_quant) once and discards them: a few loads per lane that
 * nothing waits for, so that trdq_qgemm does not start on weights that are cold in DRAM.
 * Outputs and errors are those of trdq_rotate_quant; `next` is only read. */
trdq_status trdq_rotate_quant_warm(const void *X_dev, int64_t M, int K, int64_t ldx,
                                   const float *diag_dev, int block,
                                   int8_t *Xq_dev, float *sx_dev, const trdq_weights *next, void *stream);

/* ------------------------------------ other bit-widths (the W6A6 rows of Table 3)
 * trdq_rotate_quant_warm with symmetric codes of abits bits: codes in +-(2^(abits-1) - 1), one per
 * int8, s_x[i] = max_k |V[i,k]| / (2^(abits-1) - 1).  abits = 8 is trdq_rotate_quant_warm bit for
 * bit.  trdq_prepare_weights(wbits = 6) is the weight side: per-output-channel scales and codes in
 * +-31 in the layout of wbits = 8 (trdq_weights_info reports 6, trdq_weights_export gives int8
 * codes and [N] scales).  trdq_qgemm, trdq_qgemm_asym and trdq_linear_fused take such weights
 * unchanged: the product runs on the int8 matrix instructions whatever the code width.
 * Errors as trdq_rotate_quant_warm; abits outside 2..8 -> ERR_RANGE; K > 4608 -> ERR_UNSUPPORTED. */
trdq_status trdq_rotate_quant_bits(const void *X_dev, int64_t M, int K, int64_t ldx,
                                   const float *diag_dev, int block, int abits,
                                   int8_t *Xq_dev, float *sx_dev, const trdq_weights *next, void *stream);

/* ------------------------------------ asymmetric activations (Eq. 1-3)
 * The uniform quantiser of Eq. 1-3 as printed is asymmetric: per token, s = (max - min) / 255 and
 * a zero point z, codes in 0..255, V ~ s (q - z).  The calls above use the symmetric form; this
 * pair keeps the zero point (weights stay symmetric: per output channel for wbits 8 / 6, per
 * 128-channel group and output channel for wbits 4):
 *   lo = min(min_k V, 0), hi = max(max_k V, 0), s_x = (hi - lo) / 255, z = -rint(lo / s_x),
 *   q = clamp(rint(V / s_x) + z, 0, 255);  an all-zero row gives s_x = 0, z = 0.
 * (Eq. 3 as printed lacks the minus sign; with it the zero point is the code of the value 0.)
 * Xq_dev receives q - 128 as int8 (what the matrix instruction takes) and zc_dev[i] = 128 - z_i
 * (int32 [M]); trdq_qgemm_asym adds zc[i] times the column sum of the weight codes to the integer
 * sums, which makes them sum_k (q - z) Wq exactly, then dequantises as trdq_qgemm does.
 * acc_debug_dev (optional, int32 [M, N]) receives those corrected sums.  With int4 weights the
 * zero-point term is added after the group scales, in float (zc[i] times a per-channel constant
 * prepared with the weights), and acc_debug_dev ([K/128, M, N]) receives the uncorrected group
 * sums of the stored codes q - 128.  Other arguments, layouts and errors as trdq_rotate_quant_warm /
 * trdq_qgemm; NULL zc -> ERR_NULL; K > 4608 (the quantising pass) -> ERR_UNSUPPORTED. */
trdq_status trdq_rotate_quant_asym(const void *X_dev, int64_t M, int K, int64_t ldx,
                                   const float *diag_dev, int block,
                                   int8_t *Xq_dev, float *sx_dev, int32_t *zc_dev, const trdq_weights *next,
                                   void *stream);
trdq_status trdq_qgemm_asym(const trdq_weights *w, const int8_t *Xq_dev, const float *sx_dev,
                            const int32_t *zc_dev, int64_t M, const float *bias_dev, void *Y_dev, int64_t ldy,
                            int32_t *acc_debug_dev, void *stream);

/* ------------------------------------ asymmetric weights (Eq. 1-3 on H_t(W))
 * The quantiser of Eq. 1-3 with a zero point applied to the transformed weights, one range per
 * output channel (Sec. 3.1: weights per channel), int8 storage:
 *   lo_n = min(min_k W'[k,n], 0), hi_n = max(max_k W'[k,n], 0), s_w[n] = (hi_n - lo_n) / 255,
 *   z_w[n] = -rint(lo_n / s_w[n]),  q[k,n] = clamp(rint(W'[k,n] / s_w[n]) + z_w[n], 0, 255);
 *   an all-zero channel gives s_w = 0, z_w = 0.
 * trdq_prepare_weights_asym: arguments and errors of trdq_prepare_weights; wbits must be 8
 *   (else ERR_UNSUPPORTED).  The set stores q - 128 as int8: trdq_weights_export gives those
 *   stored codes ([K, N]) and the scales, trdq_weights_export_zero_points the z_w (int32 [N] on the
 *   host; ERR_MISMATCH for a symmetric set).
 * trdq_qgemm_asym_weights: the product for such a set,
 *   acc[i,n] = sum_k (qx[i,k] - zx[i]) (q[k,n] - z_w[n])   (exact in int32; zx = 0 for symmetric codes),
 *   Y = bf16(acc * s_x[i] * s_w[n] + bias[n]).
 *   Xq_dev / sx_dev come from trdq_rotate_quant (zc_dev NULL) or from trdq_rotate_quant_asym (zc_dev
 *   its third output).  rowsum_ws_dev: int32 [M] device workspace; the call fills it with the
 *   per-token sums of the stored activation codes (a small kernel ahead of the product), which the
 *   epilogue needs for the z_w term.  acc_debug_dev (optional, int32 [M, N]) receives acc.
 *   Every other product entry point (trdq_qgemm, trdq_qgemm_asym, trdq_qgemm_tiled,
 *   trdq_linear_fused) refuses an asymmetric set with ERR_MISMATCH, and this one a symmetric set.
 *   Other arguments and errors as trdq_qgemm; NULL rowsum_ws -> ERR_NULL. */
trdq_status trdq_prepare_weights_asym(const float *W_dev, int K, int N, const float *diag_dev,
                                      int block, int wbits, void *stream, trdq_weights **out);
trdq_status trdq_weights_export_zero_points(const trdq_weights *w, int32_t *zw_host);
trdq_status trdq_qgemm_asym_weights(const trdq_weights *w, const int8_t *Xq_dev, const float *sx_dev,
                                    const int32_t *zc_dev, int32_t *rowsum_ws_dev, int64_t M,
                                    const float *bias_dev, void *Y_dev, int64_t ldy,
                                    int32_t *acc_debug_dev, void *stream);

/* ---------------------------------------------------------- calibration side
 * The per-channel statistics that the smoothing diagonal (Sec. 3.1, Eq. 5) and the zigzag
 * permutation (Sec. 3.2) are computed from, and Eq. 5 itself.  Offline, once per time-step group,
 * on calibration activations of that group. */

/* mag_dev[k] = max over the M tokens of |(X . diag)[i, k]| (rotate == 0) or of
 * |((X . diag) . R)[i, k]| (rotate != 0: after the first block rotation, the input of the zigzag
 * permutation).  X_dev, ldx, diag_dev (NULL = ones), block as in trdq_rotate_quant; mag_dev:
 * float32 [K] on the device, overwritten (M == 0 gives zeros).  Errors as trdq_rotate_quant;
 * NULL mag_dev -> ERR_NULL. */
trdq_status trdq_channel_absmax(const void *X_dev, int64_t M, int K, int64_t ldx, const float *diag_dev,
                                int rotate, int block, float *mag_dev, void *stream);

/* wmax_dev[k] = max_n |W[k, n]| for W_dev float32 [K, N] row-major (C_in x C_out): the weight side
 * of Eq. 5.  Errors: NULL -> ERR_NULL; K <= 0 or N <= 0 -> ERR_SHAPE. */
trdq_status trdq_weight_row_absmax(const float *W_dev, int K, int N, float *wmax_dev, void *stream);

/* Eq. 5 in the form this library applies it: Eq. 4 divides activations by Delta, Eq. 9/10 (and
 * every call here) multiply them by the diagonal, so diag = 1 / Delta:
 *   diag[k] = wmax[k]^(1 - alpha) / xmax[k]^alpha,   alpha in [0, 1] the migration strength;
 * a channel with xmax == 0 or wmax == 0 gets diag = 1.  All arrays float32 [K] on the device.
 * Errors: NULL -> ERR_NULL; K <= 0 -> ERR_SHAPE; alpha outside [0, 1] (or NaN) -> ERR_RANGE. */
trdq_status trdq_smooth_diag(const float *xmax_dev, const float *wmax_dev, int K, float alpha,
                             float *diag_dev, void *stream);

/* ---------------------------------------------------- dense rotation blocks
 * The BlockDiag equation of Sec. 3.2 with arbitrary orthogonal 128 x 128 blocks R_b in place of
 * the Hadamard block (for example the greedy rotations of Eq. 6-7):
 *   G_t(X) = (X . diag) . BlockDiag(R_b),   H_t(W) = BlockDiag(R_b)^T . (diag^-1 . W).
 * trdq_rotation_create copies R_dev (float32 [K/128, 128, 128], block b row-major, (k, c) = the
 * entry that takes input channel k to rotated channel c) and diag_dev (float32 [K], NULL = ones)
 * and prepares the activation-side operand; the caller's arrays may be freed afterwards.  The
 * blocks are taken as given: orthogonality is the caller's business (a non-orthogonal R changes
 * the product).  Errors: NULL -> ERR_NULL; K <= 0, K % 128 -> ERR_SHAPE; block != 128 or
 * K > 4608 -> ERR_UNSUPPORTED. */
typedef struct trdq_rotation trdq_rotation;
trdq_status trdq_rotation_create(const float *R_dev, const float *diag_dev, int K, int block, void *stream,
                                 trdq_rotation **out);
void trdq_rotation_destroy(trdq_rotation *r);

/* The greedy construction of the blocks (Eq. 6-7), block by block on calibration activations
 * X_dev (bf16 [M, K], row stride ldx) times diag_dev (NULL = ones):
 *   step k: C1 swaps column 0 with the first column holding the largest |activation| of the block,
 *           R^k = C1 Q_k C2 with C2 undoing the swap, X <- X R^k;
 *   R_b = R^1 ... R^n,  n = the first k in 1..n_steps with the smallest max|X R^1 ... R^k|.
 * Q_dev: float64 [n_steps, 128, 128] on the device, the orthogonal matrices the method draws (each
 * with a first row of equal entries; the same sequence serves every block); they are inputs.
 * R_dev: float32 [K/128, 128, 128] on the device (written: what trdq_rotation_create takes).
 * n_host: int32 [K/128] on the host (written, may be NULL).  Runs in float64; allocates its
 * workspace (8 M K bytes and a little) and synchronises the stream.
 * Errors: as trdq_rotate_quant for X; NULL Q/R -> ERR_NULL; M <= 0 or n_steps <= 0 -> ERR_SHAPE;
 * n_steps > 4096 or M K > 5e8 -> ERR_UNSUPPORTED. */
trdq_status trdq_greedy_rotation(const void *X_dev, int64_t M, int K, int64_t ldx, const float *diag_dev,
                                 int block, const double *Q_dev, int n_steps, float *R_dev, int32_t *n_host,
                                 void *stream);

/* The rest of the per-group calibration of Sec. 3.2 when the first rotation is dense:
 * trdq_channel_absmax_dense: mag_dev[k] = max_i |((X . diag) . BlockDiag(R_b))[i, k]| with the
 *   rotation's blocks and diagonal (float32 [K] on the device, overwritten): the magnitudes the
 *   zigzag permutation is dealt from.  Errors as trdq_channel_absmax.
 * trdq_greedy_rotation_second: trdq_greedy_rotation for the SECOND rotation of Eq. 10: the search runs
 *   on ((X . diag) . BlockDiag(R1))[:, perm] (computed in float64 from rot1's float32 blocks) instead
 *   of X . diag.  perm_dev int32 [K] on the device; other arguments and errors as trdq_greedy_rotation. */
trdq_status trdq_channel_absmax_dense(const void *X_dev, int64_t M, int64_t ldx, const trdq_rotation *rot,
                                      float *mag_dev, void *stream);
trdq_status trdq_greedy_rotation_second(const void *X_dev, int64_t M, int64_t ldx, const trdq_rotation *rot1,
                                        const int32_t *perm_dev, const double *Q_dev, int n_steps, float *R_dev,
                                        int32_t *n_host, void *stream);

/* trdq_prepare_weights with the rotation's blocks and diagonal (wbits 8, 6 or 4; layouts, handle
 * and errors as trdq_prepare_weights; K != the rotation's K -> ERR_MISMATCH). */
trdq_status trdq_prepare_weights_dense(const float *W_dev, int K, int N, const trdq_rotation *rot,
                                       int wbits, void *stream, trdq_weights **out);

/* trdq_rotate_quant with the rotation's blocks and diagonal: V = (X . diag) . BlockDiag(R_b),
 * then the per-token symmetric int8 quantiser.  K is the rotation's; other arguments, layouts and
 * errors as trdq_rotate_quant. */
trdq_status trdq_rotate_quant_dense(const void *X_dev, int64_t M, int64_t ldx, const trdq_rotation *rot,
                                    int8_t *Xq_dev, float *sx_dev, void *stream);

/* Eq. 10 in full with dense blocks:  G_t(X) = (X . diag) . BlockDiag(R1) . P . BlockDiag(R2)  and
 * H_t(W) = BlockDiag(R2)^T . P^T . BlockDiag(R1)^T . (diag^-1 . W).  rot1 carries the diagonal and
 * the first rotation; rot2 the second rotation and must have been created WITHOUT a diagonal
 * (else ERR_MISMATCH); perm_dev: int32 [K] on the device, (U P)[k'] = U[perm[k']] as for
 * trdq_rotate_quant_rpr.  Other arguments, layouts and errors as the one-rotation calls above;
 * the activation side takes K <= 4608 (ERR_UNSUPPORTED beyond): 16-token workgroups up to K = 1536,
 * 8-token workgroups that run the second rotation twice (maxima, then codes) for wider rows.
 * trdq_rotate_quant_dense_rpr_ws is the same operation with a device workspace, which rows wider than
 * K = 1536 (and narrower rows from 16384 tokens on) use for a faster form (a workgroup per block with the
 * rotation resident in LDS; the once-rotated values cross the permutation through the workspace as float32):
 * ws_dev holds at least trdq_rotate_quant_dense_rpr_ws_nbytes(M, K) bytes (4 (K + 1) roundup(M, 32); 0 for
 * M <= 0 and for K <= 1536 below 16384 tokens, and then ws_dev may be NULL), 16-byte aligned, and belongs to the call until it has finished on its stream;
 * nothing in it needs to be kept or cleared between calls.  ERR_NULL without it, ERR_SHAPE if it is too
 * small or misaligned, ERR_UNSUPPORTED from 2^32 workspace elements (16 GiB) on; otherwise arguments, results and errors as trdq_rotate_quant_dense_rpr (the two
 * forms round differently in the last float32 bits, so single codes may differ by one step). */
trdq_status trdq_prepare_weights_dense_rpr(const float *W_dev, int K, int N, const trdq_rotation *rot1,
                                           const int32_t *perm_dev, const trdq_rotation *rot2, int wbits,
                                           void *stream, trdq_weights **out);
trdq_status trdq_rotate_quant_dense_rpr(const void *X_dev, int64_t M, int64_t ldx, const trdq_rotation *rot1,
                                        const int32_t *perm_dev, const trdq_rotation *rot2,
                                        int8_t *Xq_dev, float *sx_dev, void *stream);
size_t trdq_rotate_quant_dense_rpr_ws_nbytes(int64_t M, int K);
trdq_status trdq_rotate_quant_dense_rpr_ws(const void *X_dev, int64_t M, int64_t ldx, const trdq_rotation *rot1,
                                           const int32_t *perm_dev, const trdq_rotation *rot2,
                                           int8_t *Xq_dev, float *sx_dev, void *ws_dev, size_t ws_bytes, void *stream);

/* ------------------------------------------------- attention sharing (Sec. 3.3)
 * Eq. 11 between the attention outputs of the conditional and the unconditional pass:
 *   cos_dev[s] = A_s . B_s / (|A_s| |B_s|)   for s < n_seg;   0 where either vector is all zero.
 * A_dev, B_dev: bf16, segment s starts at element s * stride_a (s * stride_b) and has seg_len
 * elements (16-byte aligned bases; with more than one segment the strides are multiples of 8;
 * stride >= seg_len).  acc_ws_dev: float64 [3 * n_seg] device workspace the call owns until it
 * has finished (cleared by the call).  cos_dev: float32 [n_seg].  Sums run in fp64 above 64
 * products, so the result is within 1e-5 of the exact value.  n_seg <= 65535.
 * Errors: NULL -> ERR_NULL; sizes, strides, alignment -> ERR_SHAPE. */
trdq_status trdq_cosine_similarity(const void *A_dev, const void *B_dev, int n_seg, int64_t seg_len,
                                   int64_t stride_a, int64_t stride_b, double *acc_ws_dev, float *cos_dev,
                                   void *stream);

/* The same call for callers that cannot allocate device memory or bring a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the accumulators live
 * in a fixed array inside the library, 3 float64 per segment for at most TRDQ_COSINE_STATIC_MAX_SEG
 * segments (96 KB, held by every GPU the library runs on until the process ends).  The call
 * allocates nothing, clears the accumulators it uses with a fill kernel (no memset: it may be
 * captured) and is asynchronous on `stream`.  All calls on one GPU share the array: two such calls
 * that overlap in time on one GPU (different streams, or different threads) race; callers order
 * them.  Arguments, result and accuracy as trdq_cosine_similarity.
 * Errors: NULL -> ERR_NULL; sizes, strides, alignment -> ERR_SHAPE; n_seg beyond the maximum ->
 * ERR_RANGE (before any device work). */
#define TRDQ_COSINE_STATIC_MAX_SEG 4096
trdq_status trdq_cosine_similarity_static(const void *A_dev, const void *B_dev, int n_seg, int64_t seg_len,
                                          int64_t stride_a, int64_t stride_b, float *cos_dev, void *stream);

/* Which transformer blocks share attention between the two passes: the blocks whose similarity is
 * at least `threshold` at EVERY time step (Sec. 3.3 shares the blocks that are similar across all
 * time steps).  Host arrays: sim_host float32 [n_steps, n_blocks] of Eq. 11 values, share_host
 * int32 [n_blocks] (written: 1 = share, 0 = compute both).  A NaN similarity never shares.
 * Errors: NULL -> ERR_NULL; n_steps <= 0 or n_blocks <= 0 -> ERR_SHAPE; threshold outside
 * [-1, 1] -> ERR_RANGE. */
trdq_status trdq_share_plan(const float *sim_host, int n_steps, int n_blocks, float threshold,
                            int32_t *share_host);

/* ------------------------------------------- full transform of Eq. 9
 * G_t(X) = (X . Delta_t) . R^(1) . P . R^(2)  and  H_t(W) = R^(2)^T . P^T . R^(1)^T . (Delta_t^-1 . W)
 * (Sec. 3.2: first block rotation, zigzag permutation, second block rotation).  Both rotations
 * are the block-diagonal Hadamard rotation of the calls above; the permutation is a table
 * perm[K] of source channels, (U P)[k'] = U[perm[k']], so P P^T = I and the product is unchanged.
 * Weights prepared with trdq_prepare_weights_rpr go with activations from
 * trdq_rotate_quant_rpr (same diag, same perm) through the unchanged trdq_qgemm. */

/* Zigzag permutation (Sec. 3.2): channels in order of decreasing magnitude are dealt to the
 * K / block blocks back and forth (blocks 0..nb-1, then nb-1..0, ...); round r fills slot r of
 * every block; equal magnitudes keep their channel order.  Host arrays: chan_mag_host[K] (for
 * example the per-channel absmax of calibration activations after the first rotation),
 * perm_host[K] (written).  Errors: NULL -> ERR_NULL; K <= 0, block <= 0, K % block -> ERR_SHAPE;
 * a magnitude that is NaN or infinite -> ERR_RANGE. */
trdq_status trdq_zigzag_permutation(const float *chan_mag_host, int K, int block, int32_t *perm_host);

/* trdq_prepare_weights with the permutation and the second rotation.  perm_dev: int32 [K] on the
 * device, a permutation of 0..K-1 (entries are clamped to the range, not otherwise checked).
 * Other arguments, ownership and errors as trdq_prepare_weights; NULL perm_dev -> ERR_NULL. */
trdq_status trdq_prepare_weights_rpr(const float *W_dev, int K, int N, const float *diag_dev,
                                     const int32_t *perm_dev, int block, int wbits, void *stream,
                                     trdq_weights **out);

/* trdq_rotate_quant with the permutation and the second rotation: V = (X . diag) . R . P . R,
 * then the per-token quantiser.  perm_dev as above (16-byte aligned).  K up to 4608.
 * next: as in trdq_rotate_quant_warm (the weights of the product that follows, or NULL).
 * Arguments, outputs and errors otherwise as trdq_rotate_quant; K > 4608 -> ERR_UNSUPPORTED. */
trdq_status trdq_rotate_quant_rpr(const void *X_dev, int64_t M, int K, int64_t ldx,
                                  const float *diag_dev, const int32_t *perm_dev, int block,
                                  int8_t *Xq_dev, float *sx_dev, const trdq_weights *next, void *stream);

/* trdq_rotate_quant_rpr with the asymmetric per-token quantiser of Eq. 1-3 on the fully transformed
 * activations: codes q - 128 and zc_dev[i] = 128 - z_i exactly as trdq_rotate_quant_asym writes them
 * (to be multiplied by trdq_qgemm_asym against weights from trdq_prepare_weights_rpr).
 * Errors as trdq_rotate_quant_rpr; NULL zc -> ERR_NULL. */
trdq_status trdq_rotate_quant_rpr_asym(const void *X_dev, int64_t M, int K, int64_t ldx,
                                       const float *diag_dev, const int32_t *perm_dev, int block,
                                       int8_t *Xq_dev, float *sx_dev, int32_t *zc_dev, const trdq_weights *next,
                                       void *stream);

/* The integer product G_t(X_t) . H_t(W) on the codes, with the dequantising epilogue:
 *   wbits 8: Y[i,n] = bf16( float(acc[i,n]) * s_x[i] * s_w[n] + bias[n] ),  acc = Xq . Wq  (int32, exact)
 *   wbits 4: Y[i,n] = bf16( s_x[i] * sum_g s_w[g,n] * float(acc_g[i,n]) + bias[n] ),
 *            acc_g = the partial product over input group g (int32, exact), g ascending.
 * Xq_dev: int8 [M, K] dense (16-byte aligned);  sx_dev: float32 [M];
 * bias_dev: float32 [N] or NULL;  Y_dev: bf16 [M, N], row stride ldy elements
 * (ldy >= N, ldy % 4 == 0, 8-byte aligned base).
 * acc_debug_dev: NULL, or int32 [M, N] (wbits 8) / [K/128, M, N] (wbits 4) receiving the raw
 * accumulators (for bit-exactness tests; slows the call).
 * Errors: NULL w/Xq/sx/Y -> ERR_NULL; M < 0, ldy < N, misalignment -> ERR_SHAPE. */
trdq_status trdq_qgemm(const trdq_weights *w, const int8_t *Xq_dev, const float *sx_dev, int64_t M,
                       const float *bias_dev, void *Y_dev, int64_t ldy,
                       int32_t *acc_debug_dev, void *stream);

/* ---- the same pair on block-tiled activation codes (Eq. 10's product; int8 and int4 weights) ----
 * The codes of trdq_rotate_quant in 1 KB blocks of 16 tokens x 64 input channels: code (m, k) at
 *   ((m / 16) * (K / 64) + k / 64) * 1024 + ((k % 64) / 16) * 256 + (m % 16) * 16 + k % 16
 * (inside a block, 16 bytes of k of the 16 tokens lie together: the lane order of the int8
 * matrix instruction's operand),
 * trdq_xq_tiled_nbytes(M, K) = ceil(M / 16) * 16 * K bytes (16-byte aligned; rows of a last,
 * partial group of 16 are not written).  A block is one operand fragment of the int8 matrix
 * instruction and one direct-to-LDS copy of eight whole cache lines, which lets the product run
 * 256-token tiles with two workgroups per compute unit (see qgemm_tiled.hip).
 * trdq_rotate_quant_tiled: arguments, values and errors of trdq_rotate_quant_warm; K <= 4608
 *   (wider -> ERR_UNSUPPORTED).  Codes and scales are those of trdq_rotate_quant, bit for bit.
 * trdq_xq_untile: Xq_dev [M, K] dense <- Xt_dev (for inspection and for the row-major calls).
 * trdq_qgemm_tiled: arguments, values and errors of trdq_qgemm with Xt_dev in place of Xq_dev.
 *   Takes the shapes for which trdq_qgemm_tiled_supported(w, M) is 1 -- M % 128 == 0 and either
 *   int8 weights (wbits 8 or 6) with N % 144 == 0, or int4 weights with N % 128 == 0 and at
 *   least three scale groups (K >= 384) -- and an output with ldy % 8 == 0 on a 16-byte
 *   aligned base; anything else -> ERR_UNSUPPORTED (use trdq_qgemm on row-major codes).
 *   The integer sums are those of trdq_qgemm (exact; acc_debug_dev as there, [K/128, M, N] for
 *   int4 weights), the epilogue is the same arithmetic, and so are the float folds of the int4
 *   scale groups, in the same order: the outputs are those of trdq_qgemm bit for bit.
 *   Such weight sets keep a second copy of their codes in the block form (K * N more bytes for
 *   int8, K * N / 2 for int4). */
int64_t trdq_xq_tiled_nbytes(int64_t M, int K);      /* -1 for M < 0, K <= 0 or K % 128 != 0 */
trdq_status trdq_rotate_quant_tiled(const void *X_dev, int64_t M, int K, int64_t ldx,
                                    const float *diag_dev, int block,
                                    int8_t *Xt_dev, float *sx_dev, const trdq_weights *next, void *stream);
trdq_status trdq_xq_untile(const int8_t *Xt_dev, int64_t M, int K, int8_t *Xq_dev, void *stream);
int trdq_qgemm_tiled_supported(const trdq_weights *w, int64_t M);
/* 1 where the tiled pair is also the faster one by the library's measured rule (K <= 4608 and
 * either more than one 128 x 144 output tile per compute unit, or at most one and K >= 1024;
 * int4 weights: at least one 128 x 128 tile per compute unit): what trdq_layer_forward takes by
 * itself. */
int trdq_qgemm_tiled_preferred(const trdq_weights *w, int64_t M);
trdq_status trdq_qgemm_tiled(const trdq_weights *w, const int8_t *Xt_dev, const float *sx_dev, int64_t M,
                             const float *bias_dev, void *Y_dev, int64_t ldy,
                             int32_t *acc_debug_dev, void *stream);

/* Fused variant: rotate -> quantise -> integer product -> epilogue in ONE kernel; the int8
 * activations never travel through HBM.  Same arithmetic as trdq_rotate_quant followed by
 * trdq_qgemm up to the rounding order of the fp32 rotation (an activation code may differ by
 * one LSB on a rare element, within the same tolerance).  K is taken from the handle.
 * Errors as the two calls above; K beyond the fused kernel's on-chip panel
 * (K > 6144) -> ERR_UNSUPPORTED; weights that were folded with another transform than the
 * one block rotation this kernel applies (trdq_prepare_weights_rpr, _dense, _dense_rpr)
 * -> ERR_MISMATCH. */
trdq_status trdq_linear_fused(const void *X_dev, int64_t M, int64_t ldx, const float *diag_dev,
                              const trdq_weights *w, const float *bias_dev,
                              void *Y_dev, int64_t ldy, void *stream);

/* The same kernel with the asymmetric per-token quantiser of Eq. 1-3 (the arithmetic of
 * trdq_rotate_quant_asym followed by trdq_qgemm_asym): every token gets a scale from its
 * range and a zero point, the codes and zero points stay on chip, and the epilogue adds the
 * zero-point term (128 - z_m) * colsum[n] to the integer sums before dequantising, so the
 * sums are exactly those of (q - z) * w.  Weights in the int8 layout only (8- or 6-bit codes,
 * symmetric); packed int4 weights -> ERR_UNSUPPORTED; otherwise errors as trdq_linear_fused. */
trdq_status trdq_linear_fused_asym(const void *X_dev, int64_t M, int64_t ldx, const float *diag_dev,
                                   const trdq_weights *w, const float *bias_dev,
                                   void *Y_dev, int64_t ldy, void *stream);

/* ------------------------------------------------------------------ layer
 * Convenience: one linear layer = the step table + one diagonal and one prepared
 * weight set per group (H_t depends on t, so each group keeps its own weights). */
typedef struct trdq_layer trdq_layer;

/* The layer copies the table.  Errors as above. */
trdq_status trdq_layer_create(const trdq_table *t, int K, int N, int wbits, trdq_layer **out);

/* Prepare group g from W_dev [K, N] and diag_dev [K] (or NULL = ones; the diagonal is copied
 * to a device buffer the layer owns).  Replaces an earlier setting of the same group. */
trdq_status trdq_layer_set_group(trdq_layer *l, int g, const float *diag_dev, const float *W_dev,
                                 void *stream);

/* Forward at sampling step `step`: looks up the group, then runs either the fused kernel
 * (fused > 0) or rotate_quant + qgemm through the caller's workspace (fused == 0):
 * Xq_ws_dev int8 [M, K] and sx_ws_dev float32 [M] (both may be NULL when fused > 0).
 * fused < 0 chooses: the fused kernel where it is the faster path (few tokens: one round of
 * 16-token workgroups, int8 weights, K <= 1536), else the pair, which needs the workspace.
 * X_dev bf16 [M, K] dense; Y_dev bf16 [M, N] dense.
 * Errors: step outside the table -> ERR_RANGE; group not set -> ERR_MISMATCH. */
trdq_status trdq_layer_forward(const trdq_layer *l, int step, const void *X_dev, int64_t M,
                               const float *bias_dev, void *Y_dev, int fused,
                               int8_t *Xq_ws_dev, float *sx_ws_dev, void *stream);

trdq_status trdq_layer_weights(const trdq_layer *l, int g, const trdq_weights **w_out);
void trdq_layer_destroy(trdq_layer *l);

/* --------------------------------------------------------------- selection
 * Tile-shape override for trdq_qgemm, for tuning and tests: variant < 0 restores the
 * built-in choice.  Process-wide (one atomic value: a concurrent trdq_qgemm sees the old or the
 * new choice, and every choice computes the same result).
 * Unknown variant -> ERR_RANGE. */
trdq_status trdq_qgemm_set_variant(int variant);
int trdq_qgemm_num_variants(void);

/* -------------------------------------------------------------- yardsticks
 * Two kernels that do nothing but the bounding operation of the path, for callers that report a
 * kernel's rate against what the chip delivers as well as against its published peaks.
 * Neither is part of the layer.
 *
 * trdq_peak_mfma_i8: `workgroups` workgroups of `waves` (1..8) waves; each wave issues
 * iters x 8 independent int8 16x16x64 matrix instructions from registers (operands of ones).
 * sink_dev int32 [workgroups * waves * 64] receives, per lane, the sum of its 32 accumulator
 * elements = 32 * 64 * iters (checkable; iters <= 2^20 keeps it inside int32).
 * *ops_host (may be NULL) <- operations of the launch, 2 * 16*16*64 per instruction.
 * Errors: workgroups outside 1..65536, waves outside 1..8, iters outside 1..2^20 -> ERR_RANGE.
 *
 * trdq_peak_mfma_i8_data: the same loop on operands of pseudo-random bytes.  The chip sets its clock
 * by the power it draws, and a matrix pipe draws more the more of its inputs toggle: this is the
 * yardstick for a product of quantised codes, the one above the one for the published figure.
 * Lane t of a workgroup (t = threadIdx) holds, as 16 bytes each, A fragments i = 0, 1 and B
 * fragments i = 0..3 whose 32-bit word j is h(977 t + 31 i + 7 j + 1) resp. h(131 t + 17 i + 3 j + 5),
 * h(x): x ^= x >> 16; x *= 0x7feb352d; x ^= x >> 15; x *= 0x846ca68b; x ^= x >> 16 (mod 2^32);
 * accumulator k = 0..7 multiplies A[k & 1] by B[k >> 1]; sink_dev receives, per lane, the sum of
 * its 32 accumulator elements (wrapping in int32).  Arguments and errors as trdq_peak_mfma_i8.
 *
 * trdq_peak_stream: reads n_elems 16-bit elements and writes the low byte of each (2 bytes in,
 * 1 byte out per element -- the traffic mix of trdq_rotate_quant -- with no arithmetic), 16 bytes
 * per load.  src_dev 16-byte aligned, dst_dev int8 [n_elems] 8-byte aligned, n_elems % 8 == 0
 * (else ERR_SHAPE); the two buffers must not overlap.  n_elems == 0 is a no-op.
 * Both are asynchronous on `stream` and allocate nothing. */
trdq_status trdq_peak_mfma_i8(int32_t *sink_dev, int workgroups, int waves, int iters, int64_t *ops_host,
                              void *stream);
trdq_status trdq_peak_mfma_i8_data(int32_t *sink_dev, int workgroups, int waves, int iters, int64_t *ops_host,
                                   void *stream);
trdq_status trdq_peak_stream(const void *src_dev, void *dst_dev, int64_t n_elems, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TRDQ_H */
