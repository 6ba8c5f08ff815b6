/*
 * trdq_oracle.c -- plain CPU oracle for the rotated low-bit linear of TR-DQ.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, by-the-definition
 * implementation that the GPU library is checked against.  It shares no
 * code, header, table or helper with the HIP path, and nothing in the
 * product may call it: only the tests, the smoke check and the benchmark's
 * cpu_baseline leg do.
 *
 * What it computes (paper Sec. 3.1-3.2):
 *   F_t(X_t, W) = G_t(X_t) . H_t(W)                             (Eq. 10)
 *   G_t(X) = (X . Delta_t) . R           H_t(W) = R^T . (Delta_t^-1 . W)
 * with P = I and R^(2) = I (single block rotation; the functions further down that
 * permute channels and rotate a second time add P and R^(2) of Eq. 9), R block-diagonal with
 * 2^n x 2^n blocks (the BlockDiag equation of Sec. 3.2), each block the
 * orthonormal Sylvester Hadamard matrix.  Activations are quantised per
 * token online, weights per output channel (W8) or per (input-group,
 * output channel) (W4), both with the symmetric form of the uniform
 * quantiser of Eq. 1-2 (scale = absmax / (2^(b-1)-1), no zero point,
 * nearest rounding with ties to even).
 *
 * All real arithmetic is float64.  The rotation is a dense matrix product
 * with an explicitly built R -- never a butterfly -- so a mistake in a fast
 * transform cannot be mirrored here.  No blocking, fusion or reordering
 * beyond the definitions; OpenMP only splits independent rows/columns.
 *
 * Parity pins for every function live in tests/test_oracle_*.py.  Parts that
 * no statement of the paper fixes (choice of Hadamard blocks, symmetric
 * range, int4 grouping and nibble order) are "parity unpinned" by the paper
 * and pinned only by the workload statement; they are listed in the design
 * notes.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ bf16 */

/* bf16 bit pattern -> float64, exact. */
static double bf16_bits_to_f64(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* float64 -> nearest bf16 (ties to even), in ONE rounding step.
 * bf16 = 1 sign, 8 exponent (bias 127), 7 fraction bits.  The value is
 * scaled to an integer number of bf16 quanta at its own exponent, rounded
 * with rint (round-half-even in the default FP environment), scaled back. */
uint16_t trdq_oracle_f64_to_bf16(double y)
{
    if (isnan(y)) return 0x7FC0;
    uint16_t sign = signbit(y) ? 0x8000 : 0;
    double a = fabs(y);
    if (isinf(a)) return sign | 0x7F80;
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);            /* a = m * 2^e, m in [0.5,1)  => floor(log2 a) = e-1 */
    int p = e - 1;
    if (p < -126) p = -126;        /* subnormal range shares the quantum of 2^-126 */
    double quantum = ldexp(1.0, p - 7);
    double r = rint(a / quantum);  /* exact division by a power of two */
    double v = r * quantum;        /* exactly representable as bf16 unless it overflowed */
    if (v >= ldexp(1.0, 128)) return sign | 0x7F80;
    float f = (float)v;            /* exact */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return sign | (uint16_t)(u >> 16);
}

double trdq_oracle_bf16_to_f64(uint16_t h) { return bf16_bits_to_f64(h); }

/* ------------------------------------------------------- time-step table */

/* Default step -> group map: contiguous, near-equal partition of the
 * sampling steps (the method splits the sampling process by time step and keeps
 * one set of parameters per part: abstract; t in {1..N}, Eq. 10 -- indexed here from 0). */
int trdq_oracle_table_default(int n_steps, int n_groups, int32_t *map)
{
    if (n_steps <= 0 || n_groups <= 0 || n_groups > n_steps || !map) return 1;
    for (int s = 0; s < n_steps; ++s)
        map[s] = (int32_t)(((int64_t)s * n_groups) / n_steps);
    return 0;
}

/* ------------------------------------------------------ rotation matrix */

static int popcount_u(unsigned v)
{
    int c = 0;
    while (v) { c += (int)(v & 1u); v >>= 1; }
    return c;
}

/* Sylvester Hadamard matrix of order B (power of two), natural order:
 * H[i][j] = (-1)^popcount(i & j), entries +1/-1 as int8, row-major. */
int trdq_oracle_hadamard(int B, int8_t *H)
{
    if (B <= 0 || (B & (B - 1)) || !H) return 1;
    for (int i = 0; i < B; ++i)
        for (int j = 0; j < B; ++j)
            H[(size_t)i * B + j] = (popcount_u((unsigned)i & (unsigned)j) & 1) ? -1 : 1;
    return 0;
}

/* One orthonormal block R_b = H_B / sqrt(B) as dense float64, row-major. */
static double *make_rotation_block(int B)
{
    int8_t *H = (int8_t *)malloc((size_t)B * B);
    double *R = (double *)malloc(sizeof(double) * (size_t)B * B);
    if (!H || !R) { free(H); free(R); return NULL; }
    trdq_oracle_hadamard(B, H);
    double inv = 1.0 / sqrt((double)B);
    for (size_t t = 0; t < (size_t)B * B; ++t) R[t] = (double)H[t] * inv;
    free(H);
    return R;
}

/* --------------------------------------------------- activation side G_t */

/* V = (X . diag(d)) . R   with R = BlockDiag(R_b, ..., R_b)   (Eq. 9/10, P=I, R2=I)
 * X: bf16 bit patterns [M, K] with row stride ldx; d: [K] or NULL (all ones);
 * V: float64 [M, K] dense.  Within block b, V[i, bB+j] = sum_k U[i, bB+k] R_b[k][j]. */
int trdq_oracle_rotate(const uint16_t *X, int64_t M, int K, int64_t ldx,
                       const float *d, int B, double *V)
{
    if (!X || !V || M < 0 || K <= 0 || B <= 0 || (B & (B - 1)) || K % B || ldx < K) return 1;
    double *R = make_rotation_block(B);
    if (!R) return 2;
    int nb = K / B;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        double *u = (double *)malloc(sizeof(double) * (size_t)B);
        for (int b = 0; b < nb; ++b) {
            for (int k = 0; k < B; ++k) {
                double x = bf16_bits_to_f64(X[i * ldx + (int64_t)b * B + k]);
                u[k] = d ? x * (double)d[b * B + k] : x;
            }
            for (int j = 0; j < B; ++j) {
                double s = 0.0;
                for (int k = 0; k < B; ++k) s += u[k] * R[(size_t)k * B + j];
                V[i * (int64_t)K + (int64_t)b * B + j] = s;
            }
        }
        free(u);
    }
    free(R);
    return 0;
}

/* Per-token symmetric int8 quantiser (Eq. 1-2 in symmetric form, per-token
 * granularity, scale computed online from the row's extreme value):
 *   a_i = max_k |V[i,k]|,  s_x[i] = a_i / 127,
 *   Xq[i,k] = clamp(rint(V[i,k] / s_x[i]), -127, 127);   a_i == 0 -> s=0, codes 0. */
int trdq_oracle_quant_tokens(const double *V, int64_t M, int K, int8_t *Xq, double *sx)
{
    if (!V || !Xq || !sx || M < 0 || K <= 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        const double *v = V + i * (int64_t)K;
        double a = 0.0;
        for (int k = 0; k < K; ++k) { double t = fabs(v[k]); if (t > a) a = t; }
        if (a == 0.0) {
            sx[i] = 0.0;
            for (int k = 0; k < K; ++k) Xq[i * (int64_t)K + k] = 0;
            continue;
        }
        double s = a / 127.0;
        sx[i] = s;
        for (int k = 0; k < K; ++k) {
            double q = rint(v[k] / s);
            if (q > 127.0) q = 127.0;
            if (q < -127.0) q = -127.0;
            Xq[i * (int64_t)K + k] = (int8_t)q;
        }
    }
    return 0;
}

/* The same symmetric per-token quantiser at another bit-width b (Eq. 1-2 symmetric; the paper also
 * reports W6A6, Table 3): codes in [-(2^(b-1) - 1), 2^(b-1) - 1], s_x[i] = a_i / (2^(b-1) - 1).
 * Codes are stored one per int8.  2 <= b <= 8. */
int trdq_oracle_quant_tokens_bits(const double *V, int64_t M, int K, int bits, int8_t *Xq, double *sx)
{
    if (!V || !Xq || !sx || M < 0 || K <= 0 || bits < 2 || bits > 8) return 1;
    const double qmax = (double)((1 << (bits - 1)) - 1);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        const double *v = V + i * (int64_t)K;
        double a = 0.0;
        for (int k = 0; k < K; ++k) { double t = fabs(v[k]); if (t > a) a = t; }
        double s = a / qmax;
        sx[i] = (a == 0.0) ? 0.0 : s;
        for (int k = 0; k < K; ++k) {
            double q = 0.0;
            if (a != 0.0) {
                q = rint(v[k] / s);
                if (q > qmax) q = qmax;
                if (q < -qmax) q = -qmax;
            }
            Xq[i * (int64_t)K + k] = (int8_t)q;
        }
    }
    return 0;
}

/* -------------------------------------------- asymmetric activation quantiser */

/* Per-token asymmetric 8-bit quantiser of Eq. 1-3:
 *   s_i = (hi_i - lo_i) / 255,   z_i = -rint(lo_i / s_i),   q[i,k] = clamp(rint(V[i,k] / s_i) + z_i, 0, 255),
 * so that V ~ s_i * (q - z_i).  Readings: Eq. 3 as printed has z = rint(min / s), which added in
 * Eq. 1 would map the minimum to 2 min / s; the zero point has to be the code of the value 0, hence
 * the minus sign.  The range is taken as lo = min(min_k V, 0), hi = max(max_k V, 0): zero is then
 * exactly representable, z lies in [0, 255] and a constant row has a non-zero range; a row of
 * zeros gets s = 0, z = 0 and codes 0.  Rounding: nearest, ties to even. */
int trdq_oracle_quant_tokens_asym(const double *V, int64_t M, int K, uint8_t *Xq, double *sx, int32_t *zx)
{
    if (!V || !Xq || !sx || !zx || M < 0 || K <= 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        const double *v = V + i * (int64_t)K;
        double lo = 0.0, hi = 0.0;
        for (int k = 0; k < K; ++k) { if (v[k] < lo) lo = v[k]; if (v[k] > hi) hi = v[k]; }
        if (hi == lo) {
            sx[i] = 0.0; zx[i] = 0;
            for (int k = 0; k < K; ++k) Xq[i * (int64_t)K + k] = 0;
            continue;
        }
        double s = (hi - lo) / 255.0;
        double z = -rint(lo / s);
        sx[i] = s;
        zx[i] = (int32_t)z;
        for (int k = 0; k < K; ++k) {
            double q = rint(v[k] / s) + z;
            if (q > 255.0) q = 255.0;
            if (q < 0.0) q = 0.0;
            Xq[i * (int64_t)K + k] = (uint8_t)q;
        }
    }
    return 0;
}

/* acc[i,n] = sum_k (q[i,k] - z_i) * Wq[k,n]   in int32 (|.| <= 255 * 127 * K < 2^31 for K <= 66 000):
 * the integer part of the product of the dequantised operands s_i (q - z_i) and s_w[n] Wq. */
int trdq_oracle_igemm_asym(const uint8_t *Xq, const int32_t *zx, const int8_t *Wq, int64_t M, int K, int N,
                           int32_t *acc)
{
    if (!Xq || !zx || !Wq || !acc || M < 0 || K <= 0 || N <= 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int n = 0; n < N; ++n) {
            int32_t t = 0;
            for (int k = 0; k < K; ++k)
                t += ((int32_t)Xq[i * (int64_t)K + k] - zx[i]) * (int32_t)Wq[(size_t)k * N + n];
            acc[i * (int64_t)N + n] = t;
        }
    return 0;
}

/* ------------------------------------------------ asymmetric weight quantiser */

/* Eq. 1-3 applied to the transformed weights H_t(W), one range per output channel n (Sec. 3.1:
 * weights per channel), in the reading of the activation quantiser above:
 *   lo_n = min(min_k W'[k,n], 0),  hi_n = max(max_k W'[k,n], 0),  s_n = (hi_n - lo_n) / (2^bits - 1),
 *   z_n = -rint(lo_n / s_n),  q[k,n] = clamp(rint(W'[k,n] / s_n) + z_n, 0, 2^bits - 1),  W' ~ s_n (q - z_n).
 * An all-zero column gets s = 0, z = 0, codes 0. */
int trdq_oracle_quant_weights_asym(const double *Wp, int K, int N, int bits, uint8_t *Wq, double *sw, int32_t *zw)
{
    if (!Wp || !Wq || !sw || !zw || K <= 0 || N <= 0 || bits < 2 || bits > 8) return 1;
    const double qmax = (double)((1 << bits) - 1);
    for (int n = 0; n < N; ++n) {
        double lo = 0.0, hi = 0.0;
        for (int k = 0; k < K; ++k) {
            double w = Wp[(size_t)k * N + n];
            if (w < lo) lo = w;
            if (w > hi) hi = w;
        }
        if (hi == lo) {
            sw[n] = 0.0; zw[n] = 0;
            for (int k = 0; k < K; ++k) Wq[(size_t)k * N + n] = 0;
            continue;
        }
        double s = (hi - lo) / qmax;
        double z = -rint(lo / s);
        sw[n] = s;
        zw[n] = (int32_t)z;
        for (int k = 0; k < K; ++k) {
            double q = rint(Wp[(size_t)k * N + n] / s) + z;
            if (q > qmax) q = qmax;
            if (q < 0.0) q = 0.0;
            Wq[(size_t)k * N + n] = (uint8_t)q;
        }
    }
    return 0;
}

/* acc[i,n] = sum_k (qx[i,k] - zx[i]) * (qw[k,n] - zw[n]): the integer part of the product of the
 * dequantised operands when both carry a zero point (zx may be NULL: symmetric activation codes).
 * Activation codes come as int16 so that signed (symmetric) and unsigned (asymmetric) ones fit.
 * |acc| <= 255 * 255 * K < 2^31 for K <= 33 000. */
int trdq_oracle_igemm_asym2(const int16_t *Xq, const int32_t *zx, const uint8_t *Wq, const int32_t *zw,
                            int64_t M, int K, int N, int32_t *acc)
{
    if (!Xq || !Wq || !zw || !acc || M < 0 || K <= 0 || N <= 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int n = 0; n < N; ++n) {
            int32_t t = 0;
            const int32_t z = zx ? zx[i] : 0;
            for (int k = 0; k < K; ++k)
                t += ((int32_t)Xq[i * (int64_t)K + k] - z) * ((int32_t)Wq[(size_t)k * N + n] - zw[n]);
            acc[i * (int64_t)N + n] = t;
        }
    return 0;
}

/* ------------------------------------- second rotation and zigzag permutation */

/* Zigzag permutation (Sec. 3.2, "zigzag permutation"): the channels, taken in order of
 * decreasing magnitude, are dealt one at a time to the K/B blocks: first to blocks
 * 0, 1, ..., nb-1, then back nb-1, ..., 1, 0, and so on back and forth, so that no block
 * keeps receiving the largest (or the smallest) of each round.  Round r fills slot r of
 * every block.  perm[b*B + r] = the channel placed there; as a matrix, P[perm[k'], k'] = 1,
 * i.e. (U P)[k'] = U[perm[k']].  Equal magnitudes keep their channel order. */
int trdq_oracle_zigzag(const double *mag, int K, int B, int32_t *perm)
{
    if (!mag || !perm || K <= 0 || B <= 0 || K % B) return 1;
    int nb = K / B;
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
    if (!order) return 2;
    for (int k = 0; k < K; ++k) order[k] = k;
    /* insertion sort: decreasing magnitude, stable */
    for (int t = 1; t < K; ++t) {
        int32_t c = order[t];
        int u = t - 1;
        while (u >= 0 && mag[order[u]] < mag[c]) { order[u + 1] = order[u]; --u; }
        order[u + 1] = c;
    }
    for (int r = 0; r < B; ++r)
        for (int i = 0; i < nb; ++i) {
            int b = (r % 2 == 0) ? i : nb - 1 - i;
            perm[b * B + r] = order[r * nb + i];
        }
    free(order);
    return 0;
}

/* out[i, k'] = V[i, perm[k']]   (right-multiplication by the permutation matrix P) */
int trdq_oracle_permute_cols(const double *V, int64_t M, int K, const int32_t *perm, double *out)
{
    if (!V || !perm || !out || M < 0 || K <= 0) return 1;
    for (int k = 0; k < K; ++k)
        if (perm[k] < 0 || perm[k] >= K) return 1;
    for (int64_t i = 0; i < M; ++i)
        for (int k = 0; k < K; ++k) out[i * (int64_t)K + k] = V[i * (int64_t)K + perm[k]];
    return 0;
}

/* V = U . R for float64 U [M, K]: the second block rotation R^(2) of Eq. 9, same blocks as R^(1). */
int trdq_oracle_rotate_f64(const double *U, int64_t M, int K, int B, double *V)
{
    if (!U || !V || M < 0 || K <= 0 || B <= 0 || (B & (B - 1)) || K % B) return 1;
    double *R = make_rotation_block(B);
    if (!R) return 2;
    int nb = K / B;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int b = 0; b < nb; ++b)
            for (int j = 0; j < B; ++j) {
                double s = 0.0;
                for (int k = 0; k < B; ++k) s += U[i * (int64_t)K + (int64_t)b * B + k] * R[(size_t)k * B + j];
                V[i * (int64_t)K + (int64_t)b * B + j] = s;
            }
    free(R);
    return 0;
}

/* out[k', n] = Wp[perm[k'], n]   (left-multiplication by P^T) */
int trdq_oracle_permute_rows(const double *Wp, int K, int N, const int32_t *perm, double *out)
{
    if (!Wp || !perm || !out || K <= 0 || N <= 0) return 1;
    for (int k = 0; k < K; ++k)
        if (perm[k] < 0 || perm[k] >= K) return 1;
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n) out[(size_t)k * N + n] = Wp[(size_t)perm[k] * N + n];
    return 0;
}

/* out = R^T . Wp for float64 Wp [K, N]: the (R^(2))^T factor of H_t(W) in Eq. 9. */
int trdq_oracle_rotate_rows_f64(const double *Wp, int K, int N, int B, double *out)
{
    if (!Wp || !out || K <= 0 || N <= 0 || B <= 0 || (B & (B - 1)) || K % B) return 1;
    double *R = make_rotation_block(B);
    if (!R) return 2;
    int nb = K / B;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int b = 0; b < nb; ++b)
            for (int j = 0; j < B; ++j) {
                double s = 0.0;
                for (int k = 0; k < B; ++k) s += R[(size_t)k * B + j] * Wp[(size_t)(b * B + k) * N + n];
                out[(size_t)(b * B + j) * N + n] = s;
            }
    free(R);
    return 0;
}

/* ------------------------------------------------------- weight side H_t */

/* W' = R^T . diag(1/d) . W          (H_t(W) of Eq. 10 with P=I, R2=I)
 * W: float32 [K, N] row-major (C_in x C_out as in the paper); Wp: float64 [K, N].
 * Within block b, W'[bB+j, n] = sum_k R_b[k][j] * (W[bB+k, n] / d[bB+k]). */
int trdq_oracle_rotate_weights(const float *W, int K, int N, const float *d, int B, double *Wp)
{
    if (!W || !Wp || K <= 0 || N <= 0 || B <= 0 || (B & (B - 1)) || K % B) return 1;
    double *R = make_rotation_block(B);
    if (!R) return 2;
    int nb = K / B;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        double *u = (double *)malloc(sizeof(double) * (size_t)B);
        for (int b = 0; b < nb; ++b) {
            for (int k = 0; k < B; ++k) {
                double w = (double)W[(size_t)(b * B + k) * N + n];
                u[k] = d ? (1.0 / (double)d[b * B + k]) * w : w;
            }
            for (int j = 0; j < B; ++j) {
                double s = 0.0;
                for (int k = 0; k < B; ++k) s += R[(size_t)k * B + j] * u[k];
                Wp[(size_t)(b * B + j) * N + n] = s;
            }
        }
        free(u);
    }
    free(R);
    return 0;
}

/* Symmetric weight quantiser.
 *   wbits = 8: one scale per output channel n (per-channel granularity),
 *              s_w[n] = max_k |W'[k,n]| / 127, codes in [-127,127]; sw is [N].
 *   wbits = 6: the same with 31 in place of 127 (the W6 of Table 3).
 *   wbits = 4: one scale per (input group of `group` rows, output channel),
 *              s_w[g,n] = max_{k in g} |W'[k,n]| / 7, codes in [-7,7]; sw is [K/group, N].
 * Wq: int8 [K, N], one code per byte for both widths.  Zero column/group -> scale 0, codes 0. */
int trdq_oracle_quant_weights(const double *Wp, int K, int N, int wbits, int group,
                              int8_t *Wq, double *sw)
{
    if (!Wp || !Wq || !sw || K <= 0 || N <= 0) return 1;
    if (wbits != 8 && wbits != 6 && wbits != 4) return 1;
    double qmax = (double)((1 << (wbits - 1)) - 1);          /* 127, 31, 7 */
    int glen = (wbits == 4) ? group : K;
    if (glen <= 0 || K % glen) return 1;
    int ng = K / glen;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int g = 0; g < ng; ++g) {
            double a = 0.0;
            for (int k = g * glen; k < (g + 1) * glen; ++k) {
                double t = fabs(Wp[(size_t)k * N + n]);
                if (t > a) a = t;
            }
            double s = a / qmax;
            sw[(size_t)g * N + n] = (a == 0.0) ? 0.0 : s;
            for (int k = g * glen; k < (g + 1) * glen; ++k) {
                double q = 0.0;
                if (a != 0.0) {
                    q = rint(Wp[(size_t)k * N + n] / s);
                    if (q > qmax) q = qmax;
                    if (q < -qmax) q = -qmax;
                }
                Wq[(size_t)k * N + n] = (int8_t)q;
            }
        }
    }
    return 0;
}

/* Canonical int4 packing, two codes per byte along the input dimension:
 * packed[k/2, n] = (Wq[2*(k/2), n] & 0xF) | (Wq[2*(k/2)+1, n] & 0xF) << 4   (two's complement nibbles). */
int trdq_oracle_pack_int4(const int8_t *Wq, int K, int N, uint8_t *packed)
{
    if (!Wq || !packed || K <= 0 || N <= 0 || (K & 1)) return 1;
    for (int kk = 0; kk < K / 2; ++kk)
        for (int n = 0; n < N; ++n) {
            uint8_t lo = (uint8_t)Wq[(size_t)(2 * kk) * N + n] & 0xF;
            uint8_t hi = (uint8_t)Wq[(size_t)(2 * kk + 1) * N + n] & 0xF;
            packed[(size_t)kk * N + n] = (uint8_t)(lo | (hi << 4));
        }
    return 0;
}

int trdq_oracle_unpack_int4(const uint8_t *packed, int K, int N, int8_t *Wq)
{
    if (!Wq || !packed || K <= 0 || N <= 0 || (K & 1)) return 1;
    for (int kk = 0; kk < K / 2; ++kk)
        for (int n = 0; n < N; ++n) {
            uint8_t p = packed[(size_t)kk * N + n];
            int lo = p & 0xF, hi = (p >> 4) & 0xF;
            Wq[(size_t)(2 * kk) * N + n] = (int8_t)(lo >= 8 ? lo - 16 : lo);
            Wq[(size_t)(2 * kk + 1) * N + n] = (int8_t)(hi >= 8 ? hi - 16 : hi);
        }
    return 0;
}

/* ------------------------------------------------------ integer product */

/* acc = Xq . Wq in int32, the product G_t(X_t) . H_t(W) of Eq. 10 on the codes.
 *   group == K (W8): acc is [M, N].
 *   group <  K (W4): one partial sum per input group, acc is [K/group, M, N],
 *                    acc[g, i, n] = sum_{k in group g} Xq[i,k] * Wq[k,n]. */
int trdq_oracle_igemm(const int8_t *Xq, const int8_t *Wq, int64_t M, int K, int N,
                      int group, int32_t *acc)
{
    if (!Xq || !Wq || !acc || M < 0 || K <= 0 || N <= 0 || group <= 0 || K % group) return 1;
    int ng = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int g = 0; g < ng; ++g) {
            int32_t *row = acc + ((int64_t)g * M + i) * N;
            for (int n = 0; n < N; ++n) row[n] = 0;
            for (int k = g * group; k < (g + 1) * group; ++k) {
                int32_t x = (int32_t)Xq[i * (int64_t)K + k];
                const int8_t *w = Wq + (size_t)k * N;
                for (int n = 0; n < N; ++n) row[n] += x * (int32_t)w[n];
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------- dequant */

/* Undo the two scalings of Eq. 1 and add the bias, then round to bf16:
 *   ng == 1: y = acc[i,n] * s_x[i] * s_w[n] + bias[n]
 *   ng  > 1: y = s_x[i] * sum_g (s_w[g,n] * acc[g,i,n]) + bias[n]      (g ascending)
 * Y: bf16 bit patterns [M, N]; Yd (optional): the unrounded float64 values. */
int trdq_oracle_dequant(const int32_t *acc, const double *sx, const double *sw,
                        const float *bias, int64_t M, int N, int ng,
                        uint16_t *Y, double *Yd)
{
    if (!acc || !sx || !sw || !Y || M < 0 || N <= 0 || ng <= 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int n = 0; n < N; ++n) {
            double y;
            if (ng == 1) {
                y = (double)acc[i * N + n] * sx[i] * sw[n];
            } else {
                double t = 0.0;
                for (int g = 0; g < ng; ++g)
                    t += sw[(size_t)g * N + n] * (double)acc[((int64_t)g * M + i) * N + n];
                y = sx[i] * t;
            }
            if (bias) y += (double)bias[n];
            if (Yd) Yd[i * N + n] = y;
            Y[i * N + n] = trdq_oracle_f64_to_bf16(y);
        }
    }
    return 0;
}

/* ----------------------------------------------------------- whole path */

/* One rotated linear, every step in order, for inputs already in memory.
 * Outputs that are NULL are computed into temporaries and dropped.
 * Returns 0, or a non-zero step number on failure. */
int trdq_oracle_linear(const uint16_t *X, int64_t M, int K, int64_t ldx,
                       const float *W, int N, const float *d, const float *bias,
                       int B, int wbits,
                       int8_t *Xq_out, double *sx_out, int8_t *Wq_out, double *sw_out,
                       int32_t *acc_out, uint16_t *Y)
{
    if (wbits != 8 && wbits != 4) return 1;
    int group = (wbits == 8) ? K : B;
    int ng = K / group;
    int rc = 0;
    double *V = (double *)malloc(sizeof(double) * (size_t)(M > 0 ? M : 1) * K);
    double *Wp = (double *)malloc(sizeof(double) * (size_t)K * N);
    int8_t *Xq = Xq_out ? Xq_out : (int8_t *)malloc((size_t)(M > 0 ? M : 1) * K);
    double *sx = sx_out ? sx_out : (double *)malloc(sizeof(double) * (size_t)(M > 0 ? M : 1));
    int8_t *Wq = Wq_out ? Wq_out : (int8_t *)malloc((size_t)K * N);
    double *sw = sw_out ? sw_out : (double *)malloc(sizeof(double) * (size_t)ng * N);
    int32_t *acc = acc_out ? acc_out
                           : (int32_t *)malloc(sizeof(int32_t) * (size_t)ng * (size_t)(M > 0 ? M : 1) * N);
    if (!V || !Wp || !Xq || !sx || !Wq || !sw || !acc) { rc = 100; goto done; }
    if (trdq_oracle_rotate(X, M, K, ldx, d, B, V)) { rc = 2; goto done; }
    if (trdq_oracle_quant_tokens(V, M, K, Xq, sx)) { rc = 3; goto done; }
    if (trdq_oracle_rotate_weights(W, K, N, d, B, Wp)) { rc = 4; goto done; }
    if (trdq_oracle_quant_weights(Wp, K, N, wbits, B, Wq, sw)) { rc = 4; goto done; }
    if (trdq_oracle_igemm(Xq, Wq, M, K, N, group, acc)) { rc = 5; goto done; }
    if (Y && trdq_oracle_dequant(acc, sx, sw, bias, M, N, ng, Y, NULL)) { rc = 6; goto done; }
done:
    free(V); free(Wp);
    if (!Xq_out) free(Xq);
    if (!sx_out) free(sx);
    if (!Wq_out) free(Wq);
    if (!sw_out) free(sw);
    if (!acc_out) free(acc);
    return rc;
}

#ifdef _OPENMP
#include <omp.h>
int trdq_oracle_threads(void) { return omp_get_max_threads(); }
#else
int trdq_oracle_threads(void) { return 1; }
#endif
