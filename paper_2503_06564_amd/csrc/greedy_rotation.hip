// Greedy construction of the rotation blocks (Sec. 3.2, Eq. 6-7), one block of 128 channels at a
// time and all blocks side by side (the BlockDiag equation): at step k the column with the largest
// |activation| is swapped to the front (C1), the block is multiplied by the drawn orthogonal matrix
// Q_k (first row of equal entries, which spreads that column evenly), the swap is undone (C2);
// R = R^1 ... R^n with n the first step at which max|X R^1 ... R^k| is smallest.
// Everything runs in fp64: the argmax / argmin decisions are then those of a float64 reference up
// to exact ties.  The work per step is small (a 128-wide product over the calibration tokens); the
// steps are sequential, three launches each.
#include "device_utils.h"
#include "trdq_internal.h"

namespace trdq {

namespace {

constexpr int kRows = 16;      // rows of the working matrix per workgroup in the product

// Xw[b][i][j] = X[i][b*128 + j] * d[b*128 + j];  Racc[b] = I;  best = (inf, 0)
__global__ __launch_bounds__(256) void greedy_init_kernel(const uint16_t *__restrict__ X, int64_t Mc, int nb, int64_t ldx,
                                                          const float *__restrict__ diag, double *__restrict__ Xw,
                                                          double *__restrict__ Racc, double *__restrict__ best_m,
                                                          int *__restrict__ best_n)
{
    const int b = blockIdx.y;
    const int64_t rows = Mc + kBlock;                  // the block's activations, then its accumulated rotation
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < rows * kBlock; e += (int64_t)gridDim.x * 256) {
        const int64_t i = e / kBlock;
        const int j = (int)(e % kBlock);
        if (i < Mc) {
            const double x = (double)__uint_as_float((uint32_t)X[i * ldx + b * kBlock + j] << 16);
            Xw[((int64_t)b * Mc + i) * kBlock + j] = diag ? x * (double)diag[b * kBlock + j] : x;
        } else {
            Racc[((int64_t)b * kBlock + (i - Mc)) * kBlock + j] = (i - Mc) == j ? 1.0 : 0.0;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) { best_m[b] = __longlong_as_double(0x7FF0000000000000ll); best_n[b] = 0; }
}

// The same for the SECOND rotation of Eq. 10: the working matrix starts from the activations after the
// first rotation and the permutation, Xw[b][i][j] = ((X . d) . BlockDiag(R1))[i][perm[b*128 + j]], in fp64
// on the float32 values of R1.  One workgroup per (token, block), a thread per channel.
__global__ __launch_bounds__(128) void greedy_init2_kernel(const uint16_t *__restrict__ X, int64_t Mc, int K, int64_t ldx,
                                                           const float *__restrict__ diag, const float *__restrict__ R1,
                                                           const int32_t *__restrict__ perm, double *__restrict__ Xw)
{
    const int64_t i = blockIdx.x;
    const int b = blockIdx.y, j = threadIdx.x;
    int p = perm[b * kBlock + j];
    p = p < 0 ? 0 : (p >= K ? K - 1 : p);
    const int kb = p / kBlock, c = p % kBlock;
    const uint16_t *x = X + i * ldx + kb * kBlock;
    const float *r = R1 + (size_t)kb * kBlock * kBlock + c;
    double acc = 0.0;
    for (int k = 0; k < kBlock; ++k) {
        double v = (double)__uint_as_float((uint32_t)x[k] << 16);
        if (diag) v *= (double)diag[kb * kBlock + k];
        acc = fma(v, (double)r[k * kBlock], acc);
    }
    Xw[((int64_t)b * Mc + i) * kBlock + j] = acc;
}

__global__ void greedy_clear_kernel(unsigned long long *colmax, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) colmax[i] = 0ull;
}

// colmax[b][j] = max_i |Xw[b][i][j]| (non-negative doubles order like their bit patterns)
__global__ __launch_bounds__(256) void greedy_colmax_kernel(const double *__restrict__ Xw, int64_t Mc,
                                                            unsigned long long *__restrict__ colmax)
{
    __shared__ double part[2][kBlock];
    const int b = blockIdx.y;
    const int j = threadIdx.x & 127, h = threadIdx.x >> 7;
    double m = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 2 + h; i < Mc; i += (int64_t)gridDim.x * 2)
        m = fmax(m, fabs(Xw[((int64_t)b * Mc + i) * kBlock + j]));
    part[h][j] = m;
    __syncthreads();
    if (h == 0) atomicMax(colmax + b * kBlock + j, (unsigned long long)__double_as_longlong(fmax(part[0][j], part[1][j])));
}

// One workgroup per block: the largest column maximum is max|X| after `step_done` steps; keep the
// accumulated rotation if it is the smallest so far (strictly: the first minimum), and name the
// column the next step swaps to the front (the first one holding the maximum).
__global__ __launch_bounds__(128) void greedy_pick_kernel(const unsigned long long *__restrict__ colmax, int step_done,
                                                          const double *__restrict__ Racc, double *__restrict__ Rbest,
                                                          double *__restrict__ best_m, int *__restrict__ best_n,
                                                          int *__restrict__ jstar)
{
    __shared__ double v[kBlock];
    __shared__ int keep;
    const int b = blockIdx.x, t = threadIdx.x;
    v[t] = __longlong_as_double((long long)colmax[b * kBlock + t]);
    __syncthreads();
    if (t == 0) {
        double m = v[0];
        int j = 0;
        for (int c = 1; c < kBlock; ++c)
            if (v[c] > m) { m = v[c]; j = c; }
        jstar[b] = j;
        keep = 0;
        if (step_done >= 1 && m < best_m[b]) { best_m[b] = m; best_n[b] = step_done; keep = 1; }
    }
    __syncthreads();
    if (keep)
        for (int e = t; e < kBlock * kBlock; e += 128)
            Rbest[(size_t)b * kBlock * kBlock + e] = Racc[(size_t)b * kBlock * kBlock + e];
}

// rows <- rows . C1 Q C2 for the block's activations and its accumulated rotation:
//   out[i][sigma(c)] = sum_k in[i][sigma(k)] * Q[k][c],  sigma = the swap of columns 0 and j*
__global__ __launch_bounds__(256) void greedy_apply_kernel(double *__restrict__ Xw, double *__restrict__ Racc, int64_t Mc,
                                                           const double *__restrict__ Q, const int *__restrict__ jstar)
{
    __shared__ double rows[kRows][kBlock];
    const int b = blockIdx.y;
    const int js = jstar[b];
    const int64_t total = Mc + kBlock;
    const int64_t r0 = (int64_t)blockIdx.x * kRows;
    auto row_ptr = [&](int64_t i) -> double * {
        return i < Mc ? Xw + ((int64_t)b * Mc + i) * kBlock : Racc + ((int64_t)b * kBlock + (i - Mc)) * kBlock;
    };
    for (int e = threadIdx.x; e < kRows * kBlock; e += 256) {
        const int r = e / kBlock, k = e % kBlock;
        const int src = k == 0 ? js : (k == js ? 0 : k);
        rows[r][k] = r0 + r < total ? row_ptr(r0 + r)[src] : 0.0;
    }
    __syncthreads();
    const int c = threadIdx.x & 127, h = threadIdx.x >> 7;
    double acc[kRows / 2];
#pragma unroll
    for (int r = 0; r < kRows / 2; ++r) acc[r] = 0.0;
    for (int k = 0; k < kBlock; ++k) {
        const double q = Q[k * kBlock + c];
#pragma unroll
        for (int r = 0; r < kRows / 2; ++r) acc[r] = fma(rows[h * (kRows / 2) + r][k], q, acc[r]);
    }
    const int dst = c == 0 ? js : (c == js ? 0 : c);
#pragma unroll
    for (int r = 0; r < kRows / 2; ++r) {
        const int64_t i = r0 + h * (kRows / 2) + r;
        if (i < total) row_ptr(i)[dst] = acc[r];
    }
}

__global__ void greedy_finish_kernel(const double *__restrict__ Rbest, int64_t n, float *__restrict__ R_out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) R_out[i] = (float)Rbest[i];
}

}  // namespace

// Workspace (doubles): Xw [nb][Mc][128], Racc and Rbest [nb][128][128], colmax [nb][128], best_m [nb];
// then ints: best_n [nb], jstar [nb].
size_t greedy_workspace_bytes(int64_t Mc, int K)
{
    const int nb = K / kBlock;
    return sizeof(double) * ((size_t)Mc * K + 2 * (size_t)K * kBlock + (size_t)K + nb) + sizeof(int) * 2 * (size_t)nb;
}

hipError_t launch_greedy_rotation(const uint16_t *X, int64_t Mc, int K, int64_t ldx, const float *diag,
                                  const float *R1, const int32_t *perm,
                                  const double *Q, int n_steps, void *workspace, float *R_out, int *n_out_dev,
                                  hipStream_t st)
{
    const int nb = K / kBlock;
    double *Xw = static_cast<double *>(workspace);
    double *Racc = Xw + (size_t)Mc * K;
    double *Rbest = Racc + (size_t)K * kBlock;
    unsigned long long *colmax = reinterpret_cast<unsigned long long *>(Rbest + (size_t)K * kBlock);
    double *best_m = reinterpret_cast<double *>(colmax + K);
    int *best_n = reinterpret_cast<int *>(best_m + nb);
    int *jstar = best_n + nb;

    const int64_t rows = Mc + kBlock;
    unsigned init_grid = (unsigned)((rows * kBlock + 255) / 256);
    if (init_grid > 1024) init_grid = 1024;
    hipLaunchKernelGGL(greedy_init_kernel, dim3(init_grid, nb), dim3(256), 0, st, X, Mc, nb, ldx, diag, Xw, Racc, best_m, best_n);
    if (R1)     // second rotation: replace the working activations by the rotated, permuted ones
        hipLaunchKernelGGL(greedy_init2_kernel, dim3((unsigned)Mc, nb), dim3(128), 0, st, X, Mc, K, ldx, diag, R1, perm, Xw);
    unsigned cm_grid = (unsigned)((Mc + 63) / 64);
    if (cm_grid > 64) cm_grid = 64;
    if (cm_grid < 1) cm_grid = 1;
    const unsigned ap_grid = (unsigned)((rows + kRows - 1) / kRows);
    for (int k = 0; k <= n_steps; ++k) {
        // state after k steps: column maxima, bookkeeping for step k, choice for step k + 1
        hipLaunchKernelGGL(greedy_clear_kernel, dim3((K + 255) / 256), dim3(256), 0, st, colmax, K);
        hipLaunchKernelGGL(greedy_colmax_kernel, dim3(cm_grid, nb), dim3(256), 0, st, Xw, Mc, colmax);
        hipLaunchKernelGGL(greedy_pick_kernel, dim3(nb), dim3(128), 0, st, colmax, k, Racc, Rbest, best_m, best_n, jstar);
        if (k < n_steps)
            hipLaunchKernelGGL(greedy_apply_kernel, dim3(ap_grid, nb), dim3(256), 0, st, Xw, Racc, Mc,
                               Q + (size_t)k * kBlock * kBlock, jstar);
    }
    const int64_t n = (int64_t)K * kBlock;
    hipLaunchKernelGGL(greedy_finish_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, Rbest, n, R_out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return hipMemcpyAsync(n_out_dev, best_n, sizeof(int) * nb, hipMemcpyDeviceToDevice, st);
}

}  // namespace trdq
