// Host side of libtrdq: argument validation (always before the first HIP call), the
// time-step table, weight handles, the per-layer convenience object, and the exports.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <utility>
#include <vector>

#include "trdq_internal.h"

using trdq::Table;
using trdq::Weights;

namespace trdq {

hipError_t ensure_dynamic_lds(const void *kernel, size_t bytes)
{
    static std::mutex mu;
    static std::map<std::pair<const void *, int>, size_t> set_bytes;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    size_t &cur = set_bytes[std::make_pair(kernel, dev)];
    if (bytes <= cur) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) cur = bytes;
    return e;
}

int num_cus()
{
    static std::mutex mu;
    static std::map<int, int> cus;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return 256; }
    std::lock_guard<std::mutex> lock(mu);
    auto it = cus.find(dev);
    if (it != cus.end()) return it->second;
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
        (void)hipGetLastError();
        n = 256;
    }
    cus[dev] = n;
    return n;
}

}  // namespace trdq

struct trdq_table : Table {};
struct trdq_weights : Weights {};
struct trdq_rotation : trdq::Rotation {};

struct trdq_layer {
    Table table;
    int K = 0, N = 0, wbits = 0;
    std::vector<trdq_weights *> w;     // one per group (H_t depends on t)
    std::vector<float *> diag;         // device copies of the groups' diagonals (null = ones)
    std::vector<char> set;
};

namespace {

std::atomic<int> g_variant{-1};   // test hook (trdq_qgemm_set_variant); -1 = the built-in choice

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline trdq_status hip_status(hipError_t e) { return e == hipSuccess ? TRDQ_OK : TRDQ_ERR_HIP; }

// A handle's buffers live on the device that was current when it was created.
trdq_status check_device(int handle_device)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return TRDQ_ERR_HIP;
    return dev == handle_device ? TRDQ_OK : TRDQ_ERR_MISMATCH;
}

// Data pointers may be NULL when M == 0 (an empty tensor has no storage).
trdq_status check_rotate_args(const void *X, int64_t M, int K, int64_t ldx, int block)
{
    if (block != trdq::kBlock) return TRDQ_ERR_UNSUPPORTED;
    if (M < 0 || K <= 0 || K % trdq::kBlock != 0 || ldx < K || ldx % 8 != 0) return TRDQ_ERR_SHAPE;
    if (M > 0 && !X) return TRDQ_ERR_NULL;
    if (!aligned(X, 16)) return TRDQ_ERR_SHAPE;
    return TRDQ_OK;
}

trdq_status check_out_args(const void *Y, int64_t M, int N, int64_t ldy, const float *bias)
{
    if (M < 0 || ldy < N || ldy % 4 != 0) return TRDQ_ERR_SHAPE;
    if (M > 0 && !Y) return TRDQ_ERR_NULL;
    if (!aligned(Y, 8) || (bias && !aligned(bias, 16))) return TRDQ_ERR_SHAPE;
    return TRDQ_OK;
}

}  // namespace

extern "C" {

const char *trdq_status_str(trdq_status s)
{
    switch (s) {
        case TRDQ_OK: return "ok";
        case TRDQ_ERR_NULL: return "null pointer";
        case TRDQ_ERR_SHAPE: return "bad shape, stride or alignment";
        case TRDQ_ERR_RANGE: return "index out of range";
        case TRDQ_ERR_UNSUPPORTED: return "unsupported configuration";
        case TRDQ_ERR_MISMATCH: return "handle does not match the call";
        case TRDQ_ERR_ALLOC: return "allocation failed";
        case TRDQ_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

int trdq_abi_version(void) { return 100; }

/* ------------------------------------------------------------------ table */

trdq_status trdq_table_create(int n_steps, int n_groups, const int32_t *map_host, trdq_table **out)
{
    if (!out) return TRDQ_ERR_NULL;
    *out = nullptr;
    if (n_steps <= 0 || n_groups <= 0 || n_groups > n_steps) return TRDQ_ERR_RANGE;
    if (map_host)
        for (int s = 0; s < n_steps; ++s)
            if (map_host[s] < 0 || map_host[s] >= n_groups) return TRDQ_ERR_RANGE;
    trdq_table *t = new (std::nothrow) trdq_table;
    if (!t) return TRDQ_ERR_ALLOC;
    t->map = static_cast<int32_t *>(std::malloc(sizeof(int32_t) * (size_t)n_steps));
    if (!t->map) { delete t; return TRDQ_ERR_ALLOC; }
    t->n_steps = n_steps;
    t->n_groups = n_groups;
    for (int s = 0; s < n_steps; ++s)
        t->map[s] = map_host ? map_host[s] : (int32_t)(((int64_t)s * n_groups) / n_steps);
    *out = t;
    return TRDQ_OK;
}

trdq_status trdq_table_lookup(const trdq_table *t, int step, int *group_out)
{
    if (!t || !group_out) return TRDQ_ERR_NULL;
    if (step < 0 || step >= t->n_steps) return TRDQ_ERR_RANGE;
    *group_out = t->map[step];
    return TRDQ_OK;
}

trdq_status trdq_table_sizes(const trdq_table *t, int *n_steps_out, int *n_groups_out)
{
    if (!t) return TRDQ_ERR_NULL;
    if (n_steps_out) *n_steps_out = t->n_steps;
    if (n_groups_out) *n_groups_out = t->n_groups;
    return TRDQ_OK;
}

void trdq_table_destroy(trdq_table *t)
{
    if (!t) return;
    std::free(t->map);
    delete t;
}

/* ---------------------------------------------------------------- weights */

namespace {

// Shared body of the two weight-preparation entry points.  perm_dev == nullptr: H_t(W) of Eq. 10
// with one rotation; otherwise the full H_t(W) of Eq. 9 (rotation, P^T, rotation).
trdq_status prepare_weights_impl(const float *W_dev, int K, int N, const float *diag_dev, const int32_t *perm_dev,
                                 int block, int wbits, void *stream, trdq_weights **out,
                                 const trdq::Rotation *rot = nullptr, const trdq::Rotation *rot2 = nullptr)
{
    if (!out) return TRDQ_ERR_NULL;
    *out = nullptr;
    if (!W_dev) return TRDQ_ERR_NULL;
    if (block != trdq::kBlock || (wbits != 8 && wbits != 6 && wbits != 4)) return TRDQ_ERR_UNSUPPORTED;
    if (K <= 0 || N <= 0 || K % trdq::kBlock != 0 || N % 16 != 0) return TRDQ_ERR_SHAPE;
    const int qbits = wbits;
    if (wbits == 6) wbits = 8;      // 6-bit codes live in the 8-bit layout; only the quantiser's range differs

    hipStream_t st = static_cast<hipStream_t>(stream);
    const int nb = K / trdq::kBlock;
    trdq_weights *w = new (std::nothrow) trdq_weights;
    if (!w) return TRDQ_ERR_ALLOC;
    w->K = K; w->N = N; w->wbits = wbits; w->qbits = qbits;
    w->rotation = rot ? (rot2 ? trdq::kRotDenseRPR : trdq::kRotDense) : (perm_dev ? trdq::kRotHadamardRPR : trdq::kRotHadamard);
    float *Wrot = nullptr, *Wrot2 = nullptr, *amax = nullptr;
    const size_t code_bytes = wbits == 8 ? (size_t)K * N : (size_t)K * N / 2;
    const size_t scale_count = wbits == 8 ? (size_t)N : (size_t)nb * N;
    trdq_status rc = TRDQ_OK;
    bool ok = true;
    if (hipGetDevice(&w->device) != hipSuccess) { rc = TRDQ_ERR_HIP; goto fail; }
    if (hipMalloc(&w->codes, code_bytes) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&w->scales), scale_count * sizeof(float)) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&Wrot), (size_t)K * N * sizeof(float)) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&amax), (size_t)nb * N * sizeof(float)) != hipSuccess ||
        (perm_dev && hipMalloc(reinterpret_cast<void **>(&Wrot2), (size_t)K * N * sizeof(float)) != hipSuccess) ||
        (wbits == 8 && hipMalloc(reinterpret_cast<void **>(&w->colsum), (size_t)N * sizeof(int32_t)) != hipSuccess) ||
        (wbits == 4 && hipMalloc(reinterpret_cast<void **>(&w->colsumw), (size_t)N * sizeof(float)) != hipSuccess)) {
        rc = TRDQ_ERR_ALLOC;
        goto fail;
    }
    if (rot && rot2) {
        // Eq. 10 in full with dense blocks: first rotation, rows gathered through the permutation, second rotation
        ok = trdq::launch_prepare_rotate_dense(W_dev, K, N, rot->diag, nullptr, rot->R, Wrot, amax, st) == hipSuccess &&
             trdq::launch_prepare_rotate_dense(Wrot, K, N, nullptr, perm_dev, rot2->R, Wrot2, amax, st) == hipSuccess &&
             trdq::launch_prepare_quant(Wrot2, amax, K, N, qbits, 1.0f, w->codes, w->scales, st) == hipSuccess;
    } else if (rot) {
        // dense orthonormal blocks: nothing to normalise afterwards
        ok = trdq::launch_prepare_rotate_dense(W_dev, K, N, rot->diag, nullptr, rot->R, Wrot, amax, st) == hipSuccess &&
             trdq::launch_prepare_quant(Wrot, amax, K, N, qbits, 1.0f, w->codes, w->scales, st) == hipSuccess;
    } else if (!(ok = trdq::launch_prepare_rotate(W_dev, K, N, diag_dev, nullptr, Wrot, amax, st) == hipSuccess)) {
    } else if (perm_dev) {
        // (the Hadamard form of Eq. 9)
        // rows gathered through the permutation, rotated again; two unnormalised rotations: 1/128
        ok = trdq::launch_prepare_rotate(Wrot, K, N, nullptr, perm_dev, Wrot2, amax, st) == hipSuccess &&
             trdq::launch_prepare_quant(Wrot2, amax, K, N, qbits, 0.0078125f, w->codes, w->scales, st) == hipSuccess;
    } else {
        ok = trdq::launch_prepare_quant(Wrot, amax, K, N, qbits, 0.08838834764831845f, w->codes, w->scales, st) == hipSuccess;
    }
    if (ok && wbits == 8) ok = trdq::launch_weight_colsum(w->codes, K, N, w->colsum, st) == hipSuccess;
    // widths the block-tiled product takes (whole 144-channel tiles): a second copy of the codes in 1 KB blocks
    if (ok && wbits == 8 && N % 144 == 0) {
        if (hipMalloc(&w->codes_tiled, code_bytes) != hipSuccess) { rc = TRDQ_ERR_ALLOC; goto fail; }
        ok = trdq::launch_retile_rows(static_cast<const int8_t *>(w->codes), static_cast<int8_t *>(w->codes_tiled), N, K,
                                      true, st) == hipSuccess;
    }
    if (ok && wbits == 4) ok = trdq::launch_weight_colsumw4(w->codes, w->scales, K, N, w->colsumw, st) == hipSuccess;
    // ... and of the packed int4 codes in 512-byte blocks (whole 128-channel tiles)
    if (ok && wbits == 4 && N % 128 == 0) {
        if (hipMalloc(&w->codes_tiled, code_bytes) != hipSuccess) { rc = TRDQ_ERR_ALLOC; goto fail; }
        ok = trdq::launch_retile_w4_codes(w->codes, w->codes_tiled, N, K, st) == hipSuccess;
    }
    if (!ok || hipStreamSynchronize(st) != hipSuccess) {
        rc = TRDQ_ERR_HIP;
        goto fail;
    }
    (void)hipFree(Wrot);
    if (Wrot2) (void)hipFree(Wrot2);
    (void)hipFree(amax);
    *out = w;
    return TRDQ_OK;
fail:
    (void)hipGetLastError();
    if (Wrot) (void)hipFree(Wrot);
    if (Wrot2) (void)hipFree(Wrot2);
    if (amax) (void)hipFree(amax);
    if (w->codes) (void)hipFree(w->codes);
    if (w->codes_tiled) (void)hipFree(w->codes_tiled);
    if (w->scales) (void)hipFree(w->scales);
    if (w->colsum) (void)hipFree(w->colsum);
    if (w->colsumw) (void)hipFree(w->colsumw);
    delete w;
    return rc;
}

}  // namespace

trdq_status trdq_prepare_weights(const float *W_dev, int K, int N, const float *diag_dev,
                                 int block, int wbits, void *stream, trdq_weights **out)
{
    return prepare_weights_impl(W_dev, K, N, diag_dev, nullptr, block, wbits, stream, out);
}

trdq_status trdq_prepare_weights_asym(const float *W_dev, int K, int N, const float *diag_dev,
                                      int block, int wbits, void *stream, trdq_weights **out)
{
    if (!out) return TRDQ_ERR_NULL;
    *out = nullptr;
    if (!W_dev) return TRDQ_ERR_NULL;
    if (block != trdq::kBlock || wbits != 8) return TRDQ_ERR_UNSUPPORTED;
    if (K <= 0 || N <= 0 || K % trdq::kBlock != 0 || N % 16 != 0) return TRDQ_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int nb = K / trdq::kBlock;
    trdq_weights *w = new (std::nothrow) trdq_weights;
    if (!w) return TRDQ_ERR_ALLOC;
    w->K = K; w->N = N; w->wbits = 8; w->qbits = 8;
    w->rotation = trdq::kRotHadamard;
    float *Wrot = nullptr, *amax = nullptr, *lohi = nullptr;
    trdq_status rc = TRDQ_OK;
    bool ok = true;
    if (hipGetDevice(&w->device) != hipSuccess) { rc = TRDQ_ERR_HIP; goto fail; }
    if (hipMalloc(&w->codes, (size_t)K * N) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&w->scales), (size_t)N * sizeof(float)) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&w->colsum), (size_t)N * sizeof(int32_t)) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&w->zcw), (size_t)N * sizeof(int32_t)) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&Wrot), (size_t)K * N * sizeof(float)) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&amax), (size_t)nb * N * sizeof(float)) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&lohi), (size_t)2 * N * sizeof(float)) != hipSuccess) {
        rc = TRDQ_ERR_ALLOC;
        goto fail;
    }
    ok = trdq::launch_prepare_rotate(W_dev, K, N, diag_dev, nullptr, Wrot, amax, st) == hipSuccess &&
         trdq::launch_prepare_quant_asym(Wrot, lohi, K, N, 0.08838834764831845f, w->codes, w->scales, w->zcw, st) == hipSuccess &&
         trdq::launch_weight_colsum(w->codes, K, N, w->colsum, st) == hipSuccess;
    if (!ok || hipStreamSynchronize(st) != hipSuccess) { rc = TRDQ_ERR_HIP; goto fail; }
    (void)hipFree(Wrot); (void)hipFree(amax); (void)hipFree(lohi);
    *out = w;
    return TRDQ_OK;
fail:
    (void)hipGetLastError();
    if (Wrot) (void)hipFree(Wrot);
    if (amax) (void)hipFree(amax);
    if (lohi) (void)hipFree(lohi);
    if (w->codes) (void)hipFree(w->codes);
    if (w->scales) (void)hipFree(w->scales);
    if (w->colsum) (void)hipFree(w->colsum);
    if (w->zcw) (void)hipFree(w->zcw);
    delete w;
    return rc;
}

trdq_status trdq_weights_export_zero_points(const trdq_weights *w, int32_t *zw_host)
{
    if (!w || !zw_host) return TRDQ_ERR_NULL;
    if (!w->zcw) return TRDQ_ERR_MISMATCH;
    if (hipDeviceSynchronize() != hipSuccess) return TRDQ_ERR_HIP;
    if (hipMemcpy(zw_host, w->zcw, sizeof(int32_t) * (size_t)w->N, hipMemcpyDeviceToHost) != hipSuccess) return TRDQ_ERR_HIP;
    for (int n = 0; n < w->N; ++n) zw_host[n] = 128 - zw_host[n];
    return TRDQ_OK;
}

/* ---------------------------------------------------- dense rotation blocks */

trdq_status trdq_rotation_create(const float *R_dev, const float *diag_dev, int K, int block, void *stream,
                                 trdq_rotation **out)
{
    if (!out) return TRDQ_ERR_NULL;
    *out = nullptr;
    if (!R_dev) return TRDQ_ERR_NULL;
    if (block != trdq::kBlock) return TRDQ_ERR_UNSUPPORTED;
    if (K <= 0 || K % trdq::kBlock != 0) return TRDQ_ERR_SHAPE;
    if (!trdq::rotate_quant_dense_supports(K)) return TRDQ_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    trdq_rotation *r = new (std::nothrow) trdq_rotation;
    if (!r) return TRDQ_ERR_ALLOC;
    r->K = K;
    const size_t r_bytes = (size_t)K * trdq::kBlock * sizeof(float);
    trdq_status rc = TRDQ_OK;
    if (hipGetDevice(&r->device) != hipSuccess) { rc = TRDQ_ERR_HIP; goto fail; }
    if (hipMalloc(reinterpret_cast<void **>(&r->R), r_bytes) != hipSuccess ||
        hipMalloc(&r->pieces, trdq::rotation_pieces_bytes(K)) != hipSuccess ||
        hipMalloc(&r->frags32, trdq::rotation_frags32_bytes(K)) != hipSuccess ||
        (diag_dev && hipMalloc(reinterpret_cast<void **>(&r->diag), (size_t)K * sizeof(float)) != hipSuccess)) {
        rc = TRDQ_ERR_ALLOC;
        goto fail;
    }
    if (hipMemcpyAsync(r->R, R_dev, r_bytes, hipMemcpyDeviceToDevice, st) != hipSuccess ||
        (diag_dev && hipMemcpyAsync(r->diag, diag_dev, (size_t)K * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess) ||
        trdq::launch_rotation_pieces(r->R, r->diag, K, r->pieces, st) != hipSuccess ||
        trdq::launch_rotation_frags32(r->R, K, r->frags32, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) {
        rc = TRDQ_ERR_HIP;
        goto fail;
    }
    *out = r;
    return TRDQ_OK;
fail:
    (void)hipGetLastError();
    if (r->R) (void)hipFree(r->R);
    if (r->diag) (void)hipFree(r->diag);
    if (r->pieces) (void)hipFree(r->pieces);
    if (r->frags32) (void)hipFree(r->frags32);
    delete r;
    return rc;
}

namespace {
trdq_status greedy_impl(const void *X_dev, int64_t M, int K, int64_t ldx, const float *diag_dev, int block,
                        const float *R1_dev, const int32_t *perm_dev, const double *Q_dev, int n_steps, float *R_dev,
                        int32_t *n_host, void *stream);
}

trdq_status trdq_greedy_rotation(const void *X_dev, int64_t M, int K, int64_t ldx, const float *diag_dev,
                                 int block, const double *Q_dev, int n_steps, float *R_dev, int32_t *n_host,
                                 void *stream)
{
    return greedy_impl(X_dev, M, K, ldx, diag_dev, block, nullptr, nullptr, Q_dev, n_steps, R_dev, n_host, stream);
}

trdq_status trdq_greedy_rotation_second(const void *X_dev, int64_t M, int64_t ldx, const trdq_rotation *rot1,
                                        const int32_t *perm_dev, const double *Q_dev, int n_steps, float *R_dev,
                                        int32_t *n_host, void *stream)
{
    if (!rot1 || !perm_dev) return TRDQ_ERR_NULL;
    return greedy_impl(X_dev, M, rot1->K, ldx, rot1->diag, trdq::kBlock, rot1->R, perm_dev, Q_dev, n_steps, R_dev,
                       n_host, stream);
}

trdq_status trdq_channel_absmax_dense(const void *X_dev, int64_t M, int64_t ldx, const trdq_rotation *rot,
                                      float *mag_dev, void *stream)
{
    if (!rot) return TRDQ_ERR_NULL;
    trdq_status rc = check_rotate_args(X_dev, M, rot->K, ldx, trdq::kBlock);
    if (rc != TRDQ_OK) return rc;
    if (!mag_dev) return TRDQ_ERR_NULL;
    if (!aligned(mag_dev, 4)) return TRDQ_ERR_SHAPE;
    if (trdq_status rd = check_device(rot->device); rd != TRDQ_OK) return rd;
    return hip_status(trdq::launch_channel_absmax_dense(static_cast<const uint16_t *>(X_dev), M, rot->K, ldx, rot->pieces,
                                                        mag_dev, static_cast<hipStream_t>(stream)));
}

namespace {
trdq_status greedy_impl(const void *X_dev, int64_t M, int K, int64_t ldx, const float *diag_dev, int block,
                        const float *R1_dev, const int32_t *perm_dev, const double *Q_dev, int n_steps, float *R_dev,
                        int32_t *n_host, void *stream)
{
    trdq_status rc = check_rotate_args(X_dev, M, K, ldx, block);
    if (rc != TRDQ_OK) return rc;
    if (!Q_dev || !R_dev) return TRDQ_ERR_NULL;
    if (M <= 0 || n_steps <= 0) return TRDQ_ERR_SHAPE;
    if (n_steps > 4096 || (double)M * K * 8.0 > 4.0e9) return TRDQ_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int nb = K / trdq::kBlock;
    void *ws = nullptr;
    int *n_dev = nullptr;
    if (hipMalloc(&ws, trdq::greedy_workspace_bytes(M, K)) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&n_dev), sizeof(int) * (size_t)nb) != hipSuccess) {
        (void)hipGetLastError();
        if (ws) (void)hipFree(ws);
        return TRDQ_ERR_ALLOC;
    }
    std::vector<int> n_tmp((size_t)nb, 0);
    bool ok = trdq::launch_greedy_rotation(static_cast<const uint16_t *>(X_dev), M, K, ldx, diag_dev, R1_dev, perm_dev,
                                           Q_dev, n_steps, ws, R_dev, n_dev, st) == hipSuccess &&
              hipMemcpyAsync(n_tmp.data(), n_dev, sizeof(int) * (size_t)nb, hipMemcpyDeviceToHost, st) == hipSuccess &&
              hipStreamSynchronize(st) == hipSuccess;
    (void)hipFree(ws);
    (void)hipFree(n_dev);
    if (!ok) {
        (void)hipGetLastError();
        return TRDQ_ERR_HIP;
    }
    if (n_host)
        for (int b = 0; b < nb; ++b) n_host[b] = n_tmp[(size_t)b];
    return TRDQ_OK;
}
}  // namespace

void trdq_rotation_destroy(trdq_rotation *r)
{
    if (!r) return;
    if (r->R) (void)hipFree(r->R);
    if (r->diag) (void)hipFree(r->diag);
    if (r->pieces) (void)hipFree(r->pieces);
    if (r->frags32) (void)hipFree(r->frags32);
    delete r;
}

trdq_status trdq_prepare_weights_dense(const float *W_dev, int K, int N, const trdq_rotation *rot,
                                       int wbits, void *stream, trdq_weights **out)
{
    if (out) *out = nullptr;
    if (!rot) return TRDQ_ERR_NULL;
    if (K != rot->K) return TRDQ_ERR_MISMATCH;
    return prepare_weights_impl(W_dev, K, N, nullptr, nullptr, trdq::kBlock, wbits, stream, out, rot);
}

trdq_status trdq_prepare_weights_dense_rpr(const float *W_dev, int K, int N, const trdq_rotation *rot1,
                                           const int32_t *perm_dev, const trdq_rotation *rot2, int wbits,
                                           void *stream, trdq_weights **out)
{
    if (out) *out = nullptr;
    if (!rot1 || !rot2 || !perm_dev) return TRDQ_ERR_NULL;
    if (K != rot1->K || K != rot2->K || rot2->diag) return TRDQ_ERR_MISMATCH;
    return prepare_weights_impl(W_dev, K, N, nullptr, perm_dev, trdq::kBlock, wbits, stream, out, rot1, rot2);
}

namespace {

trdq_status rotate_quant_dense_rpr_impl(const void *X_dev, int64_t M, int64_t ldx, const trdq_rotation *rot1,
                                        const int32_t *perm_dev, const trdq_rotation *rot2, int8_t *Xq_dev,
                                        float *sx_dev, bool with_ws, void *ws_dev, size_t ws_bytes, void *stream)
{
    if (!rot1 || !rot2 || !perm_dev) return TRDQ_ERR_NULL;
    if (rot1->K != rot2->K || rot2->diag) return TRDQ_ERR_MISMATCH;
    trdq_status rc = check_rotate_args(X_dev, M, rot1->K, ldx, trdq::kBlock);
    if (rc != TRDQ_OK) return rc;
    if (M > 0 && (!Xq_dev || !sx_dev)) return TRDQ_ERR_NULL;
    if (!aligned(Xq_dev, 16) || !aligned(sx_dev, 4) || !aligned(perm_dev, 4)) return TRDQ_ERR_SHAPE;
    if (!trdq::rotate_quant_dense_rpr_supports(rot1->K)) return TRDQ_ERR_UNSUPPORTED;
    const size_t need = with_ws ? trdq::rotate_quant_dense_rpr_workspace_bytes(M, rot1->K) : 0;
    if (need >= ((size_t)4 << 32)) return TRDQ_ERR_UNSUPPORTED;      // the kernels index the workspace with 32 bits
    if (need > 0) {
        if (!ws_dev) return TRDQ_ERR_NULL;
        if (!aligned(ws_dev, 16) || ws_bytes < need) return TRDQ_ERR_SHAPE;
    }
    if (M == 0) return TRDQ_OK;
    if (trdq_status rd = check_device(rot1->device); rd != TRDQ_OK) return rd;
    if (trdq_status rd = check_device(rot2->device); rd != TRDQ_OK) return rd;
    if (need > 0)
        return hip_status(trdq::launch_rotate_quant_dense_rpr_ws(static_cast<const uint16_t *>(X_dev), M, rot1->K, ldx,
                                                                 rot1->pieces, perm_dev, rot2->pieces, Xq_dev, sx_dev,
                                                                 static_cast<float *>(ws_dev),
                                                                 static_cast<hipStream_t>(stream)));
    return hip_status(trdq::launch_rotate_quant_dense_rpr(static_cast<const uint16_t *>(X_dev), M, rot1->K, ldx,
                                                          rot1->pieces, perm_dev, rot2->frags32, Xq_dev, sx_dev,
                                                          static_cast<hipStream_t>(stream)));
}

}  // namespace

trdq_status trdq_rotate_quant_dense_rpr(const void *X_dev, int64_t M, int64_t ldx, const trdq_rotation *rot1,
                                        const int32_t *perm_dev, const trdq_rotation *rot2,
                                        int8_t *Xq_dev, float *sx_dev, void *stream)
{
    return rotate_quant_dense_rpr_impl(X_dev, M, ldx, rot1, perm_dev, rot2, Xq_dev, sx_dev, false, nullptr, 0, stream);
}

size_t trdq_rotate_quant_dense_rpr_ws_nbytes(int64_t M, int K)
{
    if (M <= 0 || K <= 0 || K % trdq::kBlock != 0) return 0;
    return trdq::rotate_quant_dense_rpr_workspace_bytes(M, K);
}

trdq_status trdq_rotate_quant_dense_rpr_ws(const void *X_dev, int64_t M, int64_t ldx, const trdq_rotation *rot1,
                                           const int32_t *perm_dev, const trdq_rotation *rot2,
                                           int8_t *Xq_dev, float *sx_dev, void *ws_dev, size_t ws_bytes, void *stream)
{
    return rotate_quant_dense_rpr_impl(X_dev, M, ldx, rot1, perm_dev, rot2, Xq_dev, sx_dev, true, ws_dev, ws_bytes, stream);
}

trdq_status trdq_rotate_quant_dense(const void *X_dev, int64_t M, int64_t ldx, const trdq_rotation *rot,
                                    int8_t *Xq_dev, float *sx_dev, void *stream)
{
    if (!rot) return TRDQ_ERR_NULL;
    trdq_status rc = check_rotate_args(X_dev, M, rot->K, ldx, trdq::kBlock);
    if (rc != TRDQ_OK) return rc;
    if (M > 0 && (!Xq_dev || !sx_dev)) return TRDQ_ERR_NULL;
    if (!aligned(Xq_dev, 16) || !aligned(sx_dev, 4)) return TRDQ_ERR_SHAPE;
    if (M == 0) return TRDQ_OK;
    if (trdq_status rd = check_device(rot->device); rd != TRDQ_OK) return rd;
    return hip_status(trdq::launch_rotate_quant_dense(static_cast<const uint16_t *>(X_dev), M, rot->K, ldx, rot->pieces,
                                                      Xq_dev, sx_dev, static_cast<hipStream_t>(stream)));
}

trdq_status trdq_prepare_weights_rpr(const float *W_dev, int K, int N, const float *diag_dev,
                                     const int32_t *perm_dev, int block, int wbits, void *stream,
                                     trdq_weights **out)
{
    if (out) *out = nullptr;
    if (!perm_dev) return TRDQ_ERR_NULL;
    return prepare_weights_impl(W_dev, K, N, diag_dev, perm_dev, block, wbits, stream, out);
}

trdq_status trdq_channel_absmax(const void *X_dev, int64_t M, int K, int64_t ldx, const float *diag_dev,
                                int rotate, int block, float *mag_dev, void *stream)
{
    trdq_status rc = check_rotate_args(X_dev, M, K, ldx, block);
    if (rc != TRDQ_OK) return rc;
    if (!mag_dev) return TRDQ_ERR_NULL;
    if (!aligned(mag_dev, 4) || (diag_dev && !aligned(diag_dev, 16))) return TRDQ_ERR_SHAPE;
    return hip_status(trdq::launch_channel_absmax(static_cast<const uint16_t *>(X_dev), M, K, ldx, diag_dev,
                                                  rotate != 0, mag_dev, static_cast<hipStream_t>(stream)));
}

trdq_status trdq_weight_row_absmax(const float *W_dev, int K, int N, float *wmax_dev, void *stream)
{
    if (!W_dev || !wmax_dev) return TRDQ_ERR_NULL;
    if (K <= 0 || N <= 0) return TRDQ_ERR_SHAPE;
    return hip_status(trdq::launch_weight_row_absmax(W_dev, K, N, wmax_dev, static_cast<hipStream_t>(stream)));
}

trdq_status trdq_smooth_diag(const float *xmax_dev, const float *wmax_dev, int K, float alpha,
                             float *diag_dev, void *stream)
{
    if (!xmax_dev || !wmax_dev || !diag_dev) return TRDQ_ERR_NULL;
    if (K <= 0) return TRDQ_ERR_SHAPE;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return TRDQ_ERR_RANGE;
    return hip_status(trdq::launch_smooth_diag(xmax_dev, wmax_dev, K, alpha, diag_dev,
                                               static_cast<hipStream_t>(stream)));
}

trdq_status trdq_cosine_similarity(const void *A_dev, const void *B_dev, int n_seg, int64_t seg_len,
                                   int64_t stride_a, int64_t stride_b, double *acc_ws_dev, float *cos_dev,
                                   void *stream)
{
    if (!A_dev || !B_dev || !acc_ws_dev || !cos_dev) return TRDQ_ERR_NULL;
    if (n_seg <= 0 || n_seg > 65535 || seg_len <= 0 || stride_a < seg_len || stride_b < seg_len) return TRDQ_ERR_SHAPE;
    // 16-byte loads: bases and strides in whole 16-byte pieces (a single segment needs only the bases)
    if (!aligned(A_dev, 16) || !aligned(B_dev, 16) || !aligned(acc_ws_dev, 8) || !aligned(cos_dev, 4)) return TRDQ_ERR_SHAPE;
    if (n_seg > 1 && (stride_a % 8 != 0 || stride_b % 8 != 0)) return TRDQ_ERR_SHAPE;
    return hip_status(trdq::launch_cosine_similarity(static_cast<const uint16_t *>(A_dev),
                                                     static_cast<const uint16_t *>(B_dev), n_seg, seg_len, stride_a,
                                                     stride_b, acc_ws_dev, cos_dev, static_cast<hipStream_t>(stream)));
}

trdq_status trdq_cosine_similarity_static(const void *A_dev, const void *B_dev, int n_seg, int64_t seg_len,
                                          int64_t stride_a, int64_t stride_b, float *cos_dev, void *stream)
{
    if (!A_dev || !B_dev || !cos_dev) return TRDQ_ERR_NULL;
    if (n_seg <= 0 || seg_len <= 0 || stride_a < seg_len || stride_b < seg_len) return TRDQ_ERR_SHAPE;
    if (n_seg > trdq::kCosineStaticMaxSeg) return TRDQ_ERR_RANGE;      // beyond the fixed accumulator array
    if (!aligned(A_dev, 16) || !aligned(B_dev, 16) || !aligned(cos_dev, 4)) return TRDQ_ERR_SHAPE;
    if (n_seg > 1 && (stride_a % 8 != 0 || stride_b % 8 != 0)) return TRDQ_ERR_SHAPE;
    double *acc = nullptr;
    if (trdq::cosine_static_scratch(&acc) != hipSuccess) { (void)hipGetLastError(); return TRDQ_ERR_HIP; }
    return hip_status(trdq::launch_cosine_similarity(static_cast<const uint16_t *>(A_dev),
                                                     static_cast<const uint16_t *>(B_dev), n_seg, seg_len, stride_a,
                                                     stride_b, acc, cos_dev, static_cast<hipStream_t>(stream)));
}

static trdq_status peak_mfma_impl(int32_t *sink_dev, int workgroups, int waves, int iters, int64_t *ops_host,
                                  void *stream, bool random_data)
{
    if (!sink_dev) return TRDQ_ERR_NULL;
    if (workgroups <= 0 || workgroups > 65536 || waves <= 0 || waves > 8 || iters <= 0 || iters > (1 << 20))
        return TRDQ_ERR_RANGE;
    if (!aligned(sink_dev, 4)) return TRDQ_ERR_SHAPE;
    // one 16x16x64 instruction: 16*16*64 multiply-adds
    if (ops_host) *ops_host = (int64_t)workgroups * waves * iters * trdq::peak_mfma_independent() * 2 * 16 * 16 * 64;
    return hip_status(trdq::launch_peak_mfma_i8(sink_dev, workgroups, waves, iters, static_cast<hipStream_t>(stream),
                                                random_data));
}

trdq_status trdq_peak_mfma_i8(int32_t *sink_dev, int workgroups, int waves, int iters, int64_t *ops_host,
                              void *stream)
{
    return peak_mfma_impl(sink_dev, workgroups, waves, iters, ops_host, stream, false);
}

trdq_status trdq_peak_mfma_i8_data(int32_t *sink_dev, int workgroups, int waves, int iters, int64_t *ops_host,
                                   void *stream)
{
    return peak_mfma_impl(sink_dev, workgroups, waves, iters, ops_host, stream, true);
}

trdq_status trdq_peak_stream(const void *src_dev, void *dst_dev, int64_t n_elems, void *stream)
{
    if (n_elems < 0 || n_elems % 8 != 0) return TRDQ_ERR_SHAPE;
    if (n_elems == 0) return TRDQ_OK;
    if (!src_dev || !dst_dev) return TRDQ_ERR_NULL;
    if (!aligned(src_dev, 16) || !aligned(dst_dev, 8)) return TRDQ_ERR_SHAPE;
    return hip_status(trdq::launch_peak_stream(src_dev, dst_dev, n_elems, static_cast<hipStream_t>(stream)));
}

trdq_status trdq_share_plan(const float *sim_host, int n_steps, int n_blocks, float threshold, int32_t *share_host)
{
    if (!sim_host || !share_host) return TRDQ_ERR_NULL;
    if (n_steps <= 0 || n_blocks <= 0) return TRDQ_ERR_SHAPE;
    if (!(threshold >= -1.0f && threshold <= 1.0f)) return TRDQ_ERR_RANGE;
    for (int b = 0; b < n_blocks; ++b) {
        bool all = true;
        for (int t = 0; t < n_steps && all; ++t) all = sim_host[(size_t)t * n_blocks + b] >= threshold;   // NaN: no
        share_host[b] = all ? 1 : 0;
    }
    return TRDQ_OK;
}

trdq_status trdq_zigzag_permutation(const float *chan_mag_host, int K, int block, int32_t *perm_host)
{
    if (!chan_mag_host || !perm_host) return TRDQ_ERR_NULL;
    if (block <= 0 || K <= 0 || K % block != 0) return TRDQ_ERR_SHAPE;
    for (int k = 0; k < K; ++k)
        if (!std::isfinite(chan_mag_host[k])) return TRDQ_ERR_RANGE;   // NaN has no place in an order
    // channels by decreasing magnitude (equal magnitudes keep their order), dealt to the blocks
    // back and forth: round r fills slot r of every block, left to right on even rounds
    std::vector<int32_t> order((size_t)K);
    for (int k = 0; k < K; ++k) order[(size_t)k] = k;
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return chan_mag_host[a] > chan_mag_host[b]; });
    const int nb = K / block;
    for (int t = 0; t < K; ++t) {
        const int round = t / nb, pos = t % nb;
        const int b = (round & 1) ? nb - 1 - pos : pos;
        perm_host[b * block + round] = order[(size_t)t];
    }
    return TRDQ_OK;
}

trdq_status trdq_weights_info(const trdq_weights *w, int *K_out, int *N_out, int *wbits_out)
{
    if (!w) return TRDQ_ERR_NULL;
    if (K_out) *K_out = w->K;
    if (N_out) *N_out = w->N;
    if (wbits_out) *wbits_out = w->qbits;
    return TRDQ_OK;
}

trdq_status trdq_weights_nbytes(const trdq_weights *w, int64_t *nbytes_out)
{
    if (!w || !nbytes_out) return TRDQ_ERR_NULL;
    const int64_t codes = w->wbits == 8 ? (int64_t)w->K * w->N : (int64_t)w->K * w->N / 2;
    const int64_t scales = (w->wbits == 8 ? (int64_t)w->N : (int64_t)(w->K / trdq::kBlock) * w->N) * 4;
    *nbytes_out = codes + scales;
    return TRDQ_OK;
}

trdq_status trdq_weights_export(const trdq_weights *w, int8_t *codes_host, float *scales_host)
{
    if (!w) return TRDQ_ERR_NULL;
    const int K = w->K, N = w->N;
    if (hipDeviceSynchronize() != hipSuccess) return TRDQ_ERR_HIP;
    if (scales_host) {
        const size_t cnt = w->wbits == 8 ? (size_t)N : (size_t)(K / trdq::kBlock) * N;
        if (hipMemcpy(scales_host, w->scales, cnt * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess)
            return TRDQ_ERR_HIP;
    }
    if (codes_host) {
        const size_t bytes = w->wbits == 8 ? (size_t)K * N : (size_t)K * N / 2;
        std::vector<uint8_t> tmp;
        try { tmp.resize(bytes); } catch (...) { return TRDQ_ERR_ALLOC; }
        if (hipMemcpy(tmp.data(), w->codes, bytes, hipMemcpyDeviceToHost) != hipSuccess) return TRDQ_ERR_HIP;
        if (w->wbits == 8) {
            for (int n = 0; n < N; ++n)
                for (int k = 0; k < K; ++k)
                    codes_host[(size_t)k * N + n] = (int8_t)tmp[(size_t)n * K + k];
        } else {
            // 4 bytes hold channels k0..k0+7: byte j = code(k0+j) | code(k0+4+j) << 4
            for (int n = 0; n < N; ++n)
                for (int k0 = 0; k0 < K; k0 += 8)
                    for (int j = 0; j < 4; ++j) {
                        const uint8_t v = tmp[(size_t)n * (K / 2) + k0 / 2 + j];
                        const int lo = v & 0xF, hi = v >> 4;
                        codes_host[(size_t)(k0 + j) * N + n] = (int8_t)(lo >= 8 ? lo - 16 : lo);
                        codes_host[(size_t)(k0 + 4 + j) * N + n] = (int8_t)(hi >= 8 ? hi - 16 : hi);
                    }
        }
    }
    return TRDQ_OK;
}

trdq_status trdq_weights_export_packed(const trdq_weights *w, uint8_t *packed_host)
{
    if (!w || !packed_host) return TRDQ_ERR_NULL;
    if (w->wbits != 4) return TRDQ_ERR_MISMATCH;
    const int K = w->K, N = w->N;
    std::vector<int8_t> codes;
    try { codes.resize((size_t)K * N); } catch (...) { return TRDQ_ERR_ALLOC; }
    trdq_status rc = trdq_weights_export(w, codes.data(), nullptr);
    if (rc != TRDQ_OK) return rc;
    for (int j = 0; j < K / 2; ++j)
        for (int n = 0; n < N; ++n) {
            const uint8_t lo = (uint8_t)codes[(size_t)(2 * j) * N + n] & 0xF;
            const uint8_t hi = (uint8_t)codes[(size_t)(2 * j + 1) * N + n] & 0xF;
            packed_host[(size_t)j * N + n] = (uint8_t)(lo | (hi << 4));
        }
    return TRDQ_OK;
}

void trdq_weights_destroy(trdq_weights *w)
{
    if (!w) return;
    if (w->codes) (void)hipFree(w->codes);
    if (w->codes_tiled) (void)hipFree(w->codes_tiled);
    if (w->scales) (void)hipFree(w->scales);
    if (w->colsum) (void)hipFree(w->colsum);
    if (w->zcw) (void)hipFree(w->zcw);
    if (w->colsumw) (void)hipFree(w->colsumw);
    delete w;
}

/* ----------------------------------------------------------------- online */

trdq_status trdq_rotate_quant(const void *X_dev, int64_t M, int K, int64_t ldx,
                              const float *diag_dev, int block,
                              int8_t *Xq_dev, float *sx_dev, void *stream)
{
    return trdq_rotate_quant_warm(X_dev, M, K, ldx, diag_dev, block, Xq_dev, sx_dev, nullptr, stream);
}

trdq_status trdq_rotate_quant_warm(const void *X_dev, int64_t M, int K, int64_t ldx,
                                   const float *diag_dev, int block,
                                   int8_t *Xq_dev, float *sx_dev, const trdq_weights *next, void *stream)
{
    trdq_status rc = check_rotate_args(X_dev, M, K, ldx, block);
    if (rc != TRDQ_OK) return rc;
    if (M > 0 && (!Xq_dev || !sx_dev)) return TRDQ_ERR_NULL;
    if (!aligned(Xq_dev, 16) || !aligned(sx_dev, 4) || (diag_dev && !aligned(diag_dev, 16))) return TRDQ_ERR_SHAPE;
    if (K / trdq::kBlock > 64) return TRDQ_ERR_UNSUPPORTED;
    if (M == 0) return TRDQ_OK;
    const void *warm = nullptr;
    int64_t warm_bytes = 0;
    if (next && next->codes) {
        if (trdq_status rd = check_device(next->device); rd != TRDQ_OK) return rd;
        warm = next->codes;
        warm_bytes = (int64_t)next->N * next->K / (next->wbits == 4 ? 2 : 1);
        warm_bytes -= warm_bytes % 16;
    }
    return hip_status(trdq::launch_rotate_quant(static_cast<const uint16_t *>(X_dev), M, K, ldx, diag_dev,
                                                Xq_dev, sx_dev, nullptr, warm, warm_bytes,
                                                static_cast<hipStream_t>(stream)));
}

trdq_status trdq_rotate_quant_bits(const void *X_dev, int64_t M, int K, int64_t ldx,
                                   const float *diag_dev, int block, int abits,
                                   int8_t *Xq_dev, float *sx_dev, const trdq_weights *next, void *stream)
{
    trdq_status rc = check_rotate_args(X_dev, M, K, ldx, block);
    if (rc != TRDQ_OK) return rc;
    if (M > 0 && (!Xq_dev || !sx_dev)) return TRDQ_ERR_NULL;
    if (!aligned(Xq_dev, 16) || !aligned(sx_dev, 4) || (diag_dev && !aligned(diag_dev, 16))) return TRDQ_ERR_SHAPE;
    if (abits < 2 || abits > 8) return TRDQ_ERR_RANGE;
    if (K / trdq::kBlock > 36) return TRDQ_ERR_UNSUPPORTED;
    if (M == 0) return TRDQ_OK;
    const void *warm = nullptr;
    int64_t warm_bytes = 0;
    if (next && next->codes) {
        if (trdq_status rd = check_device(next->device); rd != TRDQ_OK) return rd;
        warm = next->codes;
        warm_bytes = (int64_t)next->N * next->K / (next->wbits == 4 ? 2 : 1);
        warm_bytes -= warm_bytes % 16;
    }
    return hip_status(trdq::launch_rotate_quant(static_cast<const uint16_t *>(X_dev), M, K, ldx, diag_dev,
                                                Xq_dev, sx_dev, nullptr, warm, warm_bytes,
                                                static_cast<hipStream_t>(stream), abits));
}

trdq_status trdq_rotate_quant_asym(const void *X_dev, int64_t M, int K, int64_t ldx,
                                   const float *diag_dev, int block,
                                   int8_t *Xq_dev, float *sx_dev, int32_t *zc_dev, const trdq_weights *next,
                                   void *stream)
{
    trdq_status rc = check_rotate_args(X_dev, M, K, ldx, block);
    if (rc != TRDQ_OK) return rc;
    if (M > 0 && (!Xq_dev || !sx_dev || !zc_dev)) return TRDQ_ERR_NULL;
    if (!aligned(Xq_dev, 16) || !aligned(sx_dev, 4) || !aligned(zc_dev, 4) || (diag_dev && !aligned(diag_dev, 16)))
        return TRDQ_ERR_SHAPE;
    if (K / trdq::kBlock > 36) return TRDQ_ERR_UNSUPPORTED;
    if (M == 0) return TRDQ_OK;
    const void *warm = nullptr;
    int64_t warm_bytes = 0;
    if (next && next->codes) {
        if (trdq_status rd = check_device(next->device); rd != TRDQ_OK) return rd;
        warm = next->codes;
        warm_bytes = (int64_t)next->N * next->K / (next->wbits == 4 ? 2 : 1);
        warm_bytes -= warm_bytes % 16;
    }
    return hip_status(trdq::launch_rotate_quant(static_cast<const uint16_t *>(X_dev), M, K, ldx, diag_dev,
                                                Xq_dev, sx_dev, zc_dev, warm, warm_bytes,
                                                static_cast<hipStream_t>(stream)));
}

trdq_status trdq_rotate_quant_rpr(const void *X_dev, int64_t M, int K, int64_t ldx,
                                  const float *diag_dev, const int32_t *perm_dev, int block,
                                  int8_t *Xq_dev, float *sx_dev, const trdq_weights *next, void *stream)
{
    trdq_status rc = check_rotate_args(X_dev, M, K, ldx, block);
    if (rc != TRDQ_OK) return rc;
    if (!perm_dev) return TRDQ_ERR_NULL;
    if (M > 0 && (!Xq_dev || !sx_dev)) return TRDQ_ERR_NULL;
    if (!aligned(Xq_dev, 16) || !aligned(sx_dev, 4) || !aligned(perm_dev, 16) || (diag_dev && !aligned(diag_dev, 16)))
        return TRDQ_ERR_SHAPE;
    if (!trdq::rotate_quant_rpr_supports(K)) return TRDQ_ERR_UNSUPPORTED;
    if (M == 0) return TRDQ_OK;
    const void *warm = nullptr;
    int64_t warm_bytes = 0;
    if (next && next->codes) {
        if (trdq_status rd = check_device(next->device); rd != TRDQ_OK) return rd;
        warm = next->codes;
        warm_bytes = (int64_t)next->N * next->K / (next->wbits == 4 ? 2 : 1);
        warm_bytes -= warm_bytes % 16;
    }
    return hip_status(trdq::launch_rotate_quant_rpr(static_cast<const uint16_t *>(X_dev), M, K, ldx, diag_dev,
                                                    perm_dev, Xq_dev, sx_dev, warm, warm_bytes,
                                                    static_cast<hipStream_t>(stream)));
}

int64_t trdq_xq_tiled_nbytes(int64_t M, int K)
{
    if (M < 0 || K <= 0 || K % trdq::kBlock != 0) return -1;
    return (M + 15) / 16 * 16 * (int64_t)K;
}

trdq_status trdq_rotate_quant_tiled(const void *X_dev, int64_t M, int K, int64_t ldx,
                                    const float *diag_dev, int block,
                                    int8_t *Xt_dev, float *sx_dev, const trdq_weights *next, void *stream)
{
    trdq_status rc = check_rotate_args(X_dev, M, K, ldx, block);
    if (rc != TRDQ_OK) return rc;
    if (M > 0 && (!Xt_dev || !sx_dev)) return TRDQ_ERR_NULL;
    if (!aligned(Xt_dev, 16) || !aligned(sx_dev, 4) || (diag_dev && !aligned(diag_dev, 16))) return TRDQ_ERR_SHAPE;
    if (K / trdq::kBlock > 36) return TRDQ_ERR_UNSUPPORTED;
    if (M == 0) return TRDQ_OK;
    const void *warm = nullptr;
    int64_t warm_bytes = 0;
    if (next && next->codes) {
        if (trdq_status rd = check_device(next->device); rd != TRDQ_OK) return rd;
        // warm what the tiled product will read
        warm = next->codes_tiled ? next->codes_tiled : next->codes;
        warm_bytes = (int64_t)next->N * next->K / (next->wbits == 4 ? 2 : 1);
        warm_bytes -= warm_bytes % 16;
    }
    return hip_status(trdq::launch_rotate_quant(static_cast<const uint16_t *>(X_dev), M, K, ldx, diag_dev,
                                                Xt_dev, sx_dev, nullptr, warm, warm_bytes,
                                                static_cast<hipStream_t>(stream), 8, true));
}

trdq_status trdq_xq_untile(const int8_t *Xt_dev, int64_t M, int K, int8_t *Xq_dev, void *stream)
{
    if (M < 0 || K <= 0 || K % trdq::kBlock != 0) return TRDQ_ERR_SHAPE;
    if (M > 0 && (!Xt_dev || !Xq_dev)) return TRDQ_ERR_NULL;
    if (!aligned(Xt_dev, 16) || !aligned(Xq_dev, 16)) return TRDQ_ERR_SHAPE;
    if (M == 0) return TRDQ_OK;
    return hip_status(trdq::launch_retile_rows(Xt_dev, Xq_dev, M, K, false, static_cast<hipStream_t>(stream)));
}

int trdq_qgemm_tiled_supported(const trdq_weights *w, int64_t M)
{
    if (!w || M < 0) return 0;
    // (the output checks of the call itself, alignment and row stride, are not part of this answer)
    if (!w->codes_tiled || M % 128 != 0) return 0;
    if (w->wbits == 4) return w->N % 128 == 0 && w->K % 128 == 0 && w->K >= 384 ? 1 : 0;
    return w->wbits == 8 && w->N % 144 == 0 && w->K % 64 == 0 ? 1 : 0;
}

int trdq_qgemm_tiled_preferred(const trdq_weights *w, int64_t M)
{
    if (!trdq_qgemm_tiled_supported(w, M) || w->K / trdq::kBlock > 36) return 0;
    // int4 weights: measured 5-15 % ahead of the row-major kernel from one 128 x 128 tile per compute unit on
    if (w->wbits == 4) return (M / 128) * (int64_t)(w->N / 128) >= trdq::num_cus() ? 1 : 0;
    return trdq::qgemm_tiled_pays(M, w->K, w->N) ? 1 : 0;
}

trdq_status trdq_qgemm_tiled(const trdq_weights *w, const int8_t *Xt_dev, const float *sx_dev, int64_t M,
                             const float *bias_dev, void *Y_dev, int64_t ldy,
                             int32_t *acc_debug_dev, void *stream)
{
    if (!w) return TRDQ_ERR_NULL;
    trdq_status rc = check_out_args(Y_dev, M, w->N, ldy, bias_dev);
    if (rc != TRDQ_OK) return rc;
    if (M > 0 && (!Xt_dev || !sx_dev)) return TRDQ_ERR_NULL;
    if (!aligned(Xt_dev, 16) || !aligned(sx_dev, 4) || (acc_debug_dev && !aligned(acc_debug_dev, 16)))
        return TRDQ_ERR_SHAPE;
    if (!trdq_qgemm_tiled_supported(w, M) || ldy % 8 != 0 || !aligned(Y_dev, 16)) return TRDQ_ERR_UNSUPPORTED;
    if (M == 0) return TRDQ_OK;
    if (trdq_status rd = check_device(w->device); rd != TRDQ_OK) return rd;
    return hip_status(trdq::launch_qgemm_tiled(*w, Xt_dev, sx_dev, M, bias_dev, static_cast<uint16_t *>(Y_dev), ldy,
                                               acc_debug_dev, static_cast<hipStream_t>(stream)));
}

trdq_status trdq_rotate_quant_rpr_asym(const void *X_dev, int64_t M, int K, int64_t ldx,
                                       const float *diag_dev, const int32_t *perm_dev, int block,
                                       int8_t *Xq_dev, float *sx_dev, int32_t *zc_dev, const trdq_weights *next,
                                       void *stream)
{
    trdq_status rc = check_rotate_args(X_dev, M, K, ldx, block);
    if (rc != TRDQ_OK) return rc;
    if (!perm_dev) return TRDQ_ERR_NULL;
    if (M > 0 && (!Xq_dev || !sx_dev || !zc_dev)) return TRDQ_ERR_NULL;
    if (!aligned(Xq_dev, 16) || !aligned(sx_dev, 4) || !aligned(zc_dev, 4) || !aligned(perm_dev, 16) ||
        (diag_dev && !aligned(diag_dev, 16)))
        return TRDQ_ERR_SHAPE;
    if (!trdq::rotate_quant_rpr_supports(K)) return TRDQ_ERR_UNSUPPORTED;
    if (M == 0) return TRDQ_OK;
    const void *warm = nullptr;
    int64_t warm_bytes = 0;
    if (next && next->codes) {
        if (trdq_status rd = check_device(next->device); rd != TRDQ_OK) return rd;
        warm = next->codes;
        warm_bytes = (int64_t)next->N * next->K / (next->wbits == 4 ? 2 : 1);
        warm_bytes -= warm_bytes % 16;
    }
    return hip_status(trdq::launch_rotate_quant_rpr(static_cast<const uint16_t *>(X_dev), M, K, ldx, diag_dev,
                                                    perm_dev, Xq_dev, sx_dev, warm, warm_bytes,
                                                    static_cast<hipStream_t>(stream), zc_dev));
}

trdq_status trdq_qgemm(const trdq_weights *w, const int8_t *Xq_dev, const float *sx_dev, int64_t M,
                       const float *bias_dev, void *Y_dev, int64_t ldy,
                       int32_t *acc_debug_dev, void *stream)
{
    if (!w) return TRDQ_ERR_NULL;
    trdq_status rc = check_out_args(Y_dev, M, w->N, ldy, bias_dev);
    if (rc != TRDQ_OK) return rc;
    if (M > 0 && (!Xq_dev || !sx_dev)) return TRDQ_ERR_NULL;
    if (!aligned(Xq_dev, 16) || !aligned(sx_dev, 4) || (acc_debug_dev && !aligned(acc_debug_dev, 16)))
        return TRDQ_ERR_SHAPE;
    if (w->zcw) return TRDQ_ERR_MISMATCH;       // asymmetric weights need the row sums: trdq_qgemm_asym_weights
    if (M == 0) return TRDQ_OK;
    if (trdq_status rd = check_device(w->device); rd != TRDQ_OK) return rd;
    return hip_status(trdq::launch_qgemm(*w, Xq_dev, sx_dev, nullptr, M, bias_dev, static_cast<uint16_t *>(Y_dev), ldy,
                                         acc_debug_dev, g_variant.load(std::memory_order_relaxed), static_cast<hipStream_t>(stream)));
}

trdq_status trdq_qgemm_asym_weights(const trdq_weights *w, const int8_t *Xq_dev, const float *sx_dev,
                                    const int32_t *zc_dev, int32_t *rowsum_ws_dev, int64_t M,
                                    const float *bias_dev, void *Y_dev, int64_t ldy,
                                    int32_t *acc_debug_dev, void *stream)
{
    if (!w) return TRDQ_ERR_NULL;
    trdq_status rc = check_out_args(Y_dev, M, w->N, ldy, bias_dev);
    if (rc != TRDQ_OK) return rc;
    if (M > 0 && (!Xq_dev || !sx_dev || !rowsum_ws_dev)) return TRDQ_ERR_NULL;
    if (!aligned(Xq_dev, 16) || !aligned(sx_dev, 4) || !aligned(rowsum_ws_dev, 4) || (zc_dev && !aligned(zc_dev, 4)) ||
        (acc_debug_dev && !aligned(acc_debug_dev, 16)))
        return TRDQ_ERR_SHAPE;
    if (!w->zcw) return TRDQ_ERR_MISMATCH;
    if (M == 0) return TRDQ_OK;
    if (trdq_status rd = check_device(w->device); rd != TRDQ_OK) return rd;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (trdq::launch_xq_rowsum(Xq_dev, M, w->K, rowsum_ws_dev, st) != hipSuccess) { (void)hipGetLastError(); return TRDQ_ERR_HIP; }
    return hip_status(trdq::launch_qgemm(*w, Xq_dev, sx_dev, zc_dev, M, bias_dev, static_cast<uint16_t *>(Y_dev), ldy,
                                         acc_debug_dev, -1, st, rowsum_ws_dev));
}

trdq_status trdq_qgemm_asym(const trdq_weights *w, const int8_t *Xq_dev, const float *sx_dev,
                            const int32_t *zc_dev, int64_t M, const float *bias_dev, void *Y_dev, int64_t ldy,
                            int32_t *acc_debug_dev, void *stream)
{
    if (!w) return TRDQ_ERR_NULL;
    trdq_status rc = check_out_args(Y_dev, M, w->N, ldy, bias_dev);
    if (rc != TRDQ_OK) return rc;
    if (M > 0 && (!Xq_dev || !sx_dev || !zc_dev)) return TRDQ_ERR_NULL;
    if (!aligned(Xq_dev, 16) || !aligned(sx_dev, 4) || !aligned(zc_dev, 4) ||
        (acc_debug_dev && !aligned(acc_debug_dev, 16)))
        return TRDQ_ERR_SHAPE;
    if (w->zcw) return TRDQ_ERR_MISMATCH;       // asymmetric weights: trdq_qgemm_asym_weights
    if (M == 0) return TRDQ_OK;
    if (trdq_status rd = check_device(w->device); rd != TRDQ_OK) return rd;
    return hip_status(trdq::launch_qgemm(*w, Xq_dev, sx_dev, zc_dev, M, bias_dev, static_cast<uint16_t *>(Y_dev), ldy,
                                         acc_debug_dev, -1, static_cast<hipStream_t>(stream)));
}

static trdq_status linear_fused_impl(const void *X_dev, int64_t M, int64_t ldx, const float *diag_dev,
                                     const trdq_weights *w, const float *bias_dev,
                                     void *Y_dev, int64_t ldy, void *stream, bool asym)
{
    if (!w) return TRDQ_ERR_NULL;
    trdq_status rc = check_rotate_args(X_dev, M, w->K, ldx, trdq::kBlock);
    if (rc != TRDQ_OK) return rc;
    rc = check_out_args(Y_dev, M, w->N, ldy, bias_dev);
    if (rc != TRDQ_OK) return rc;
    if (diag_dev && !aligned(diag_dev, 16)) return TRDQ_ERR_SHAPE;
    if (!trdq::fused_supports(w->K)) return TRDQ_ERR_UNSUPPORTED;
    if (w->rotation != trdq::kRotHadamard) return TRDQ_ERR_MISMATCH;   // the kernel applies the one-rotation transform
    if (w->zcw) return TRDQ_ERR_MISMATCH;                              // ... and no zero points of the weights
    if (asym && w->wbits != 8) return TRDQ_ERR_UNSUPPORTED;            // zero points of the tokens: int8 layout only
    if (M == 0) return TRDQ_OK;
    if (trdq_status rd = check_device(w->device); rd != TRDQ_OK) return rd;
    return hip_status(trdq::launch_linear_fused(*w, static_cast<const uint16_t *>(X_dev), M, ldx, diag_dev,
                                                bias_dev, static_cast<uint16_t *>(Y_dev), ldy,
                                                static_cast<hipStream_t>(stream), asym));
}

trdq_status trdq_linear_fused(const void *X_dev, int64_t M, int64_t ldx, const float *diag_dev,
                              const trdq_weights *w, const float *bias_dev,
                              void *Y_dev, int64_t ldy, void *stream)
{
    return linear_fused_impl(X_dev, M, ldx, diag_dev, w, bias_dev, Y_dev, ldy, stream, false);
}

trdq_status trdq_linear_fused_asym(const void *X_dev, int64_t M, int64_t ldx, const float *diag_dev,
                                   const trdq_weights *w, const float *bias_dev,
                                   void *Y_dev, int64_t ldy, void *stream)
{
    return linear_fused_impl(X_dev, M, ldx, diag_dev, w, bias_dev, Y_dev, ldy, stream, true);
}

/* ------------------------------------------------------------------ layer */

trdq_status trdq_layer_create(const trdq_table *t, int K, int N, int wbits, trdq_layer **out)
{
    if (!out) return TRDQ_ERR_NULL;
    *out = nullptr;
    if (!t) return TRDQ_ERR_NULL;
    if (wbits != 8 && wbits != 6 && wbits != 4) return TRDQ_ERR_UNSUPPORTED;
    if (K <= 0 || N <= 0 || K % trdq::kBlock != 0 || N % 16 != 0) return TRDQ_ERR_SHAPE;
    trdq_layer *l = new (std::nothrow) trdq_layer;
    if (!l) return TRDQ_ERR_ALLOC;
    l->table.n_steps = t->n_steps;
    l->table.n_groups = t->n_groups;
    l->table.map = static_cast<int32_t *>(std::malloc(sizeof(int32_t) * (size_t)t->n_steps));
    if (!l->table.map) { delete l; return TRDQ_ERR_ALLOC; }
    std::memcpy(l->table.map, t->map, sizeof(int32_t) * (size_t)t->n_steps);
    l->K = K; l->N = N; l->wbits = wbits;
    try {
        l->w.assign((size_t)t->n_groups, nullptr);
        l->diag.assign((size_t)t->n_groups, nullptr);
        l->set.assign((size_t)t->n_groups, 0);
    } catch (...) {
        std::free(l->table.map);
        delete l;
        return TRDQ_ERR_ALLOC;
    }
    *out = l;
    return TRDQ_OK;
}

trdq_status trdq_layer_set_group(trdq_layer *l, int g, const float *diag_dev, const float *W_dev, void *stream)
{
    if (!l || !W_dev) return TRDQ_ERR_NULL;
    if (g < 0 || g >= l->table.n_groups) return TRDQ_ERR_RANGE;
    if (diag_dev && !aligned(diag_dev, 16)) return TRDQ_ERR_SHAPE;
    trdq_weights *w = nullptr;
    trdq_status rc = trdq_prepare_weights(W_dev, l->K, l->N, diag_dev, trdq::kBlock, l->wbits, stream, &w);
    if (rc != TRDQ_OK) return rc;
    float *d = nullptr;
    if (diag_dev) {
        if (hipMalloc(reinterpret_cast<void **>(&d), sizeof(float) * (size_t)l->K) != hipSuccess) {
            trdq_weights_destroy(w);
            return TRDQ_ERR_ALLOC;
        }
        if (hipMemcpy(d, diag_dev, sizeof(float) * (size_t)l->K, hipMemcpyDeviceToDevice) != hipSuccess) {
            (void)hipFree(d);
            trdq_weights_destroy(w);
            return TRDQ_ERR_HIP;
        }
    }
    if (l->w[(size_t)g]) trdq_weights_destroy(l->w[(size_t)g]);
    if (l->diag[(size_t)g]) (void)hipFree(l->diag[(size_t)g]);
    l->w[(size_t)g] = w;
    l->diag[(size_t)g] = d;
    l->set[(size_t)g] = 1;
    return TRDQ_OK;
}

trdq_status trdq_layer_forward(const trdq_layer *l, int step, const void *X_dev, int64_t M,
                               const float *bias_dev, void *Y_dev, int fused,
                               int8_t *Xq_ws_dev, float *sx_ws_dev, void *stream)
{
    if (!l) return TRDQ_ERR_NULL;
    if (step < 0 || step >= l->table.n_steps) return TRDQ_ERR_RANGE;
    const int g = l->table.map[step];
    if (!l->set[(size_t)g]) return TRDQ_ERR_MISMATCH;
    const trdq_weights *w = l->w[(size_t)g];
    const float *d = l->diag[(size_t)g];
    if (fused > 0 || (fused < 0 && trdq::fused_pays(M, l->K, l->N, w->wbits)))
        return trdq_linear_fused(X_dev, M, l->K, d, w, bias_dev, Y_dev, l->N, stream);
    if (!Xq_ws_dev || !sx_ws_dev) return TRDQ_ERR_NULL;
    // the workspace is private to the layer: block-tiled codes where the tiled product takes the shape
    // (M % 128 == 0 there, so the workspace size M * K is the same)
    if (trdq_qgemm_tiled_preferred(w, M) && aligned(Y_dev, 16)) {
        trdq_status rt = trdq_rotate_quant_tiled(X_dev, M, l->K, l->K, d, trdq::kBlock, Xq_ws_dev, sx_ws_dev, w, stream);
        if (rt != TRDQ_OK) return rt;
        return trdq_qgemm_tiled(w, Xq_ws_dev, sx_ws_dev, M, bias_dev, Y_dev, l->N, nullptr, stream);
    }
    trdq_status rc = trdq_rotate_quant_warm(X_dev, M, l->K, l->K, d, trdq::kBlock, Xq_ws_dev, sx_ws_dev, w, stream);
    if (rc != TRDQ_OK) return rc;
    return trdq_qgemm(w, Xq_ws_dev, sx_ws_dev, M, bias_dev, Y_dev, l->N, nullptr, stream);
}

trdq_status trdq_layer_weights(const trdq_layer *l, int g, const trdq_weights **w_out)
{
    if (!l || !w_out) return TRDQ_ERR_NULL;
    if (g < 0 || g >= l->table.n_groups) return TRDQ_ERR_RANGE;
    if (!l->set[(size_t)g]) return TRDQ_ERR_MISMATCH;
    *w_out = l->w[(size_t)g];
    return TRDQ_OK;
}

void trdq_layer_destroy(trdq_layer *l)
{
    if (!l) return;
    for (trdq_weights *w : l->w) trdq_weights_destroy(w);
    for (float *d : l->diag)
        if (d) (void)hipFree(d);
    std::free(l->table.map);
    delete l;
}

/* --------------------------------------------------------------- selection */

trdq_status trdq_qgemm_set_variant(int variant)
{
    if (variant >= trdq::qgemm_num_variants()) return TRDQ_ERR_RANGE;
    g_variant.store(variant < 0 ? -1 : variant, std::memory_order_relaxed);
    return TRDQ_OK;
}

int trdq_qgemm_num_variants(void) { return trdq::qgemm_num_variants(); }

}  // extern "C"
