"""ctypes front end of the C oracle (oracle/trdq_oracle.c).

TEST INFRASTRUCTURE ONLY: argument marshalling around the plain C functions,
plus `acc_exact_blas`, the same integer product evaluated through a float64
library matmul (every partial sum is an integer below 2^53, hence exact),
used where the plain loop would take minutes.  The steps follow Eq. 1-2
(symmetric form), the BlockDiag rotation and Eq. 9/10 of the paper, with
P = I and R^(2) = I in the basic path and with the zigzag permutation and the
second rotation in the *_rpr functions.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        i64, i32, p = C.c_int64, C.c_int, C.c_void_p
        L.trdq_oracle_f64_to_bf16.restype = C.c_uint16
        L.trdq_oracle_f64_to_bf16.argtypes = [C.c_double]
        L.trdq_oracle_bf16_to_f64.restype = C.c_double
        L.trdq_oracle_bf16_to_f64.argtypes = [C.c_uint16]
        L.trdq_oracle_table_default.argtypes = [i32, i32, p]
        L.trdq_oracle_hadamard.argtypes = [i32, p]
        L.trdq_oracle_rotate.argtypes = [p, i64, i32, i64, p, i32, p]
        L.trdq_oracle_quant_tokens.argtypes = [p, i64, i32, p, p]
        L.trdq_oracle_quant_tokens_bits.argtypes = [p, i64, i32, i32, p, p]
        L.trdq_oracle_rotate_weights.argtypes = [p, i32, i32, p, i32, p]
        L.trdq_oracle_quant_weights.argtypes = [p, i32, i32, i32, i32, p, p]
        L.trdq_oracle_pack_int4.argtypes = [p, i32, i32, p]
        L.trdq_oracle_unpack_int4.argtypes = [p, i32, i32, p]
        L.trdq_oracle_igemm.argtypes = [p, p, i64, i32, i32, i32, p]
        L.trdq_oracle_dequant.argtypes = [p, p, p, p, i64, i32, i32, p, p]
        L.trdq_oracle_linear.argtypes = [p, i64, i32, i64, p, i32, p, p, i32, i32,
                                         p, p, p, p, p, p]
        L.trdq_oracle_quant_tokens_asym.argtypes = [p, i64, i32, p, p, p]
        L.trdq_oracle_igemm_asym.argtypes = [p, p, p, i64, i32, i32, p]
        L.trdq_oracle_quant_weights_asym.argtypes = [p, i32, i32, i32, p, p, p]
        L.trdq_oracle_igemm_asym2.argtypes = [p, p, p, p, i64, i32, i32, p]
        L.trdq_oracle_zigzag.argtypes = [p, i32, i32, p]
        L.trdq_oracle_permute_cols.argtypes = [p, i64, i32, p, p]
        L.trdq_oracle_rotate_f64.argtypes = [p, i64, i32, i32, p]
        L.trdq_oracle_permute_rows.argtypes = [p, i32, i32, p, p]
        L.trdq_oracle_rotate_rows_f64.argtypes = [p, i32, i32, i32, p]
        L.trdq_oracle_threads.restype = i32
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def _c(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def threads():
    return int(lib().trdq_oracle_threads())


def f64_to_bf16(y):
    y = np.asarray(y, dtype=np.float64)
    out = np.empty(y.shape, dtype=np.uint16)
    f = lib().trdq_oracle_f64_to_bf16
    flat_in, flat_out = y.reshape(-1), out.reshape(-1)
    for t in range(flat_in.size):
        flat_out[t] = f(float(flat_in[t]))
    return out


def bf16_to_f64(h):
    h = np.asarray(h, dtype=np.uint16)
    return (h.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def table_default(n_steps, n_groups):
    m = np.empty(n_steps, dtype=np.int32)
    _chk(lib().trdq_oracle_table_default(n_steps, n_groups, _ptr(m)), "table_default")
    return m


def hadamard(B):
    H = np.empty((B, B), dtype=np.int8)
    _chk(lib().trdq_oracle_hadamard(B, _ptr(H)), "hadamard")
    return H


def rotate(X_bf16, d=None, B=128):
    """V = (X diag(d)) R as float64; X_bf16 is a uint16 [M, K] array of bf16 bit patterns."""
    X = _c(X_bf16, np.uint16)
    M, K = X.shape
    d = _c(d, np.float32)
    V = np.empty((M, K), dtype=np.float64)
    _chk(lib().trdq_oracle_rotate(_ptr(X), M, K, K, _ptr(d), B, _ptr(V)), "rotate")
    return V


def quant_tokens(V, abits=8):
    """Per-token symmetric quantiser; abits = 8 is the path's own, other widths (Table 3's A6) go
    through the general routine."""
    V = _c(V, np.float64)
    M, K = V.shape
    Xq = np.empty((M, K), dtype=np.int8)
    sx = np.empty(M, dtype=np.float64)
    if abits == 8:
        _chk(lib().trdq_oracle_quant_tokens(_ptr(V), M, K, _ptr(Xq), _ptr(sx)), "quant_tokens")
    else:
        _chk(lib().trdq_oracle_quant_tokens_bits(_ptr(V), M, K, int(abits), _ptr(Xq), _ptr(sx)), "quant_tokens_bits")
    return Xq, sx


def quant_tokens_bits(V, abits):
    """The general routine at any width 2..8 (also 8: the pins compare it with quant_tokens)."""
    V = _c(V, np.float64)
    M, K = V.shape
    Xq = np.empty((M, K), dtype=np.int8)
    sx = np.empty(M, dtype=np.float64)
    _chk(lib().trdq_oracle_quant_tokens_bits(_ptr(V), M, K, int(abits), _ptr(Xq), _ptr(sx)), "quant_tokens_bits")
    return Xq, sx


def rotate_quant(X_bf16, d=None, B=128, abits=8):
    return quant_tokens(rotate(X_bf16, d, B), abits)


def rotate_weights(W, d=None, B=128):
    W = _c(W, np.float32)
    K, N = W.shape
    d = _c(d, np.float32)
    Wp = np.empty((K, N), dtype=np.float64)
    _chk(lib().trdq_oracle_rotate_weights(_ptr(W), K, N, _ptr(d), B, _ptr(Wp)), "rotate_weights")
    return Wp


def quant_weights(Wp, wbits=8, group=128):
    Wp = _c(Wp, np.float64)
    K, N = Wp.shape
    ng = K // group if wbits == 4 else 1
    Wq = np.empty((K, N), dtype=np.int8)
    sw = np.empty((ng, N), dtype=np.float64)
    _chk(lib().trdq_oracle_quant_weights(_ptr(Wp), K, N, wbits, group, _ptr(Wq), _ptr(sw)),
         "quant_weights")
    return Wq, (sw if wbits == 4 else sw[0])


def prepare_weights(W, d=None, B=128, wbits=8):
    return quant_weights(rotate_weights(W, d, B), wbits, B)


# ---- full G_t / H_t of Eq. 9: first rotation, zigzag permutation, second rotation ----------

def zigzag(mag, B=128):
    """Zigzag permutation of Sec. 3.2 from per-channel magnitudes; perm[k'] = source channel."""
    mag = _c(mag, np.float64)
    K = mag.shape[0]
    perm = np.empty(K, dtype=np.int32)
    _chk(lib().trdq_oracle_zigzag(_ptr(mag), K, B, _ptr(perm)), "zigzag")
    return perm


def permute_cols(V, perm):
    V = _c(V, np.float64)
    M, K = V.shape
    perm = _c(perm, np.int32)
    out = np.empty((M, K), dtype=np.float64)
    _chk(lib().trdq_oracle_permute_cols(_ptr(V), M, K, _ptr(perm), _ptr(out)), "permute_cols")
    return out


def rotate_f64(U, B=128):
    U = _c(U, np.float64)
    M, K = U.shape
    V = np.empty((M, K), dtype=np.float64)
    _chk(lib().trdq_oracle_rotate_f64(_ptr(U), M, K, B, _ptr(V)), "rotate_f64")
    return V


def rotate_rpr(X_bf16, d, perm, B=128):
    """V = (X diag(d)) R P R as float64 (G_t of Eq. 9)."""
    return rotate_f64(permute_cols(rotate(X_bf16, d, B), perm), B)


def rotate_quant_rpr(X_bf16, d, perm, B=128):
    return quant_tokens(rotate_rpr(X_bf16, d, perm, B))


def rotate_weights_rpr(W, d, perm, B=128):
    """W' = R^T P^T R^T diag(1/d) W as float64 (H_t of Eq. 9)."""
    W1 = rotate_weights(W, d, B)
    K, N = W1.shape
    perm = _c(perm, np.int32)
    W2 = np.empty((K, N), dtype=np.float64)
    _chk(lib().trdq_oracle_permute_rows(_ptr(W1), K, N, _ptr(perm), _ptr(W2)), "permute_rows")
    W3 = np.empty((K, N), dtype=np.float64)
    _chk(lib().trdq_oracle_rotate_rows_f64(_ptr(W2), K, N, B, _ptr(W3)), "rotate_rows_f64")
    return W3


def prepare_weights_rpr(W, d, perm, B=128, wbits=8):
    return quant_weights(rotate_weights_rpr(W, d, perm, B), wbits, B)


def linear_rpr(X_bf16, W, d, perm, bias=None, B=128, wbits=8, exact_blas=False):
    """Whole path with the full G_t and H_t of Eq. 9."""
    Xq, sx = rotate_quant_rpr(X_bf16, d, perm, B)
    Wq, sw = prepare_weights_rpr(W, d, perm, B, wbits)
    group = None if wbits == 8 else B
    acc = (acc_exact_blas if exact_blas else igemm)(Xq, Wq, group)
    Y, Yd = dequant(acc, sx, sw, bias, return_f64=True)
    return dict(Xq=Xq, sx=sx, Wq=Wq, sw=sw, acc=acc, Y=Y, Yd=Yd)


# ---- asymmetric per-token activation quantiser (Eq. 1-3 with a zero point) --------------------

def quant_tokens_asym(V):
    """(codes uint8 [M, K] in 0..255, scales float64 [M], zero points int32 [M]); V ~ s (q - z)."""
    V = _c(V, np.float64)
    M, K = V.shape
    Xq = np.empty((M, K), dtype=np.uint8)
    sx = np.empty(M, dtype=np.float64)
    zx = np.empty(M, dtype=np.int32)
    _chk(lib().trdq_oracle_quant_tokens_asym(_ptr(V), M, K, _ptr(Xq), _ptr(sx), _ptr(zx)), "quant_tokens_asym")
    return Xq, sx, zx


def igemm_asym(Xq, zx, Wq):
    """int32 [M, N]: sum_k (q[i,k] - z_i) Wq[k,n], the plain loop."""
    Xq, zx, Wq = _c(Xq, np.uint8), _c(zx, np.int32), _c(Wq, np.int8)
    M, K = Xq.shape
    N = Wq.shape[1]
    acc = np.empty((M, N), dtype=np.int32)
    _chk(lib().trdq_oracle_igemm_asym(_ptr(Xq), _ptr(zx), _ptr(Wq), M, K, N, _ptr(acc)), "igemm_asym")
    return acc


def acc_asym_exact_blas(Xq, zx, Wq):
    """The same sums through a float64 library matmul (all partial sums are integers below 2^53)."""
    Xd = np.asarray(Xq).astype(np.float64) - np.asarray(zx).astype(np.float64)[:, None]
    return (Xd @ np.asarray(Wq).astype(np.float64)).astype(np.int32)


def igemm_asym_groups(Xq, zx, Wq, group, exact_blas=False):
    """int32 [K/group, M, N]: the sums of igemm_asym per group of `group` input channels (the int4
    weights carry one scale per group and output channel)."""
    Xq, zx, Wq = _c(Xq, np.uint8), _c(zx, np.int32), _c(Wq, np.int8)
    K = Xq.shape[1]
    f = acc_asym_exact_blas if exact_blas else igemm_asym
    return np.stack([f(Xq[:, k0:k0 + group], zx, Wq[k0:k0 + group]) for k0 in range(0, K, group)])


def linear_asym(X_bf16, W, d=None, bias=None, B=128, exact_blas=False, wbits=8):
    """Rotated linear with asymmetric per-token activations (Eq. 1-3); weights stay symmetric, per
    output channel (wbits 8, 6) or per group of B input channels and output channel (wbits 4)."""
    V = rotate(X_bf16, d, B)
    Xq, sx, zx = quant_tokens_asym(V)
    Wq, sw = prepare_weights(W, d, B, wbits)
    if wbits == 4:
        acc = igemm_asym_groups(Xq, zx, Wq, B, exact_blas)
    else:
        acc = acc_asym_exact_blas(Xq, zx, Wq) if exact_blas else igemm_asym(Xq, zx, Wq)
    Y, Yd = dequant(acc, sx, sw, bias, return_f64=True)
    return dict(Xq=Xq, sx=sx, zx=zx, Wq=Wq, sw=sw, acc=acc, Y=Y, Yd=Yd)


# ---- asymmetric weights (Eq. 1-3 applied to H_t(W), one range per output channel) --------------

def quant_weights_asym(Wp, bits=8):
    """(codes uint8 [K, N] in 0..2^bits-1, scales float64 [N], zero points int32 [N]); W' ~ s (q - z)."""
    Wp = _c(Wp, np.float64)
    K, N = Wp.shape
    Wq = np.empty((K, N), dtype=np.uint8)
    sw = np.empty(N, dtype=np.float64)
    zw = np.empty(N, dtype=np.int32)
    _chk(lib().trdq_oracle_quant_weights_asym(_ptr(Wp), K, N, bits, _ptr(Wq), _ptr(sw), _ptr(zw)), "quant_weights_asym")
    return Wq, sw, zw


def prepare_weights_asym(W, d=None, B=128, bits=8):
    return quant_weights_asym(rotate_weights(W, d, B), bits)


def igemm_asym2(Xq, zx, Wq, zw):
    """int32 [M, N]: sum_k (qx[i,k] - zx_i) (qw[k,n] - zw_n), the plain loop; zx None = symmetric activation codes."""
    Xq, zx, Wq, zw = _c(Xq, np.int16), _c(zx, np.int32), _c(Wq, np.uint8), _c(zw, np.int32)
    M, K = Xq.shape
    N = Wq.shape[1]
    acc = np.empty((M, N), dtype=np.int32)
    _chk(lib().trdq_oracle_igemm_asym2(_ptr(Xq), _ptr(zx), _ptr(Wq), _ptr(zw), M, K, N, _ptr(acc)), "igemm_asym2")
    return acc


def acc_asym2_exact_blas(Xq, zx, Wq, zw):
    """The same sums through a float64 library matmul (all partial sums are integers below 2^53)."""
    Xd = np.asarray(Xq).astype(np.float64)
    if zx is not None:
        Xd = Xd - np.asarray(zx).astype(np.float64)[:, None]
    Wd = np.asarray(Wq).astype(np.float64) - np.asarray(zw).astype(np.float64)[None, :]
    return (Xd @ Wd).astype(np.int32)


def linear_asym_weights(X_bf16, W, d=None, bias=None, B=128, exact_blas=False, act_asym=False, wbits=8):
    """Rotated linear with asymmetric per-output-channel weights (Eq. 1-3 on H_t(W)); activations
    symmetric per token, or asymmetric too (act_asym)."""
    V = rotate(X_bf16, d, B)
    if act_asym:
        Xq, sx, zx = quant_tokens_asym(V)
    else:
        Xq, sx = quant_tokens(V)
        zx = None
    Wq, sw, zw = prepare_weights_asym(W, d, B, wbits)
    f = acc_asym2_exact_blas if exact_blas else igemm_asym2
    acc = f(Xq, zx, Wq, zw)
    Y, Yd = dequant(acc, sx, sw, bias, return_f64=True)
    return dict(Xq=Xq, sx=sx, zx=zx, Wq=Wq, sw=sw, zw=zw, acc=acc, Y=Y, Yd=Yd)


def linear_rpr_asym(X_bf16, W, d, perm, bias=None, B=128, exact_blas=False):
    """The full G_t of Eq. 9 followed by the asymmetric per-token quantiser of Eq. 1-3; weights as linear_rpr (int8)."""
    Xq, sx, zx = quant_tokens_asym(rotate_rpr(X_bf16, d, perm, B))
    Wq, sw = prepare_weights_rpr(W, d, perm, B, 8)
    acc = acc_asym_exact_blas(Xq, zx, Wq) if exact_blas else igemm_asym(Xq, zx, Wq)
    Y, Yd = dequant(acc, sx, sw, bias, return_f64=True)
    return dict(Xq=Xq, sx=sx, zx=zx, Wq=Wq, sw=sw, acc=acc, Y=Y, Yd=Yd)


# ---- calibration side: Eq. 5 and the statistics it and the zigzag permutation need ----------

# ---- greedy dense block rotations (Sec. 3.2, Eq. 6-7 and the BlockDiag equation) ---------------

def greedy_rotation(Xb, Qs):
    """The rotation of ONE block by the greedy strategy of Eq. 6-7.

    Xb: float64 [Mc, B] calibration activations of the block (after the diagonal).
    Qs: float64 [N, B, B] the orthogonal matrices the method draws, one per step (each with a
        first row of equal magnitudes); they are inputs, not generated here.
    Step k: C1 swaps column 0 with the column that holds the largest |activation|, R^k = C1 Q_k C2
    with C2 swapping the two columns back (Eq. 6); X <- X R^k.  R = R^1 ... R^n with
    n = argmin_k max|X R^1 ... R^k| over k = 1..N (Eq. 7; the first minimum).
    Returns (R [B, B], n, m) with m[k-1] = max|X R^1 ... R^k|."""
    X = np.array(Xb, dtype=np.float64)
    Qs = np.asarray(Qs, dtype=np.float64)
    B = X.shape[1]
    R = np.eye(B)
    best_R, best_m, best_n = None, np.inf, 0
    m = np.empty(len(Qs))
    for k, Q in enumerate(Qs, start=1):
        j = int(np.argmax(np.abs(X).max(axis=0)))          # first column holding the largest outlier
        C1 = np.eye(B)
        C1[:, [0, j]] = C1[:, [j, 0]]
        Rk = C1 @ Q @ C1                                    # C2 = C1: the same swap undoes it
        X = X @ Rk
        R = R @ Rk
        m[k - 1] = np.abs(X).max()
        if m[k - 1] < best_m:
            best_R, best_m, best_n = R.copy(), m[k - 1], k
    return best_R, best_n, m


def greedy_rotations(X_bf16, d, Qs, B=128):
    """Eq. 6-7 block by block (the BlockDiag equation): R [K/B, B, B], n [K/B], on calibration
    activations X (bf16 bits [Mc, K]) times the diagonal d."""
    U = bf16_to_f64(_c(X_bf16, np.uint16))
    if d is not None:
        U = U * np.asarray(d, dtype=np.float32).astype(np.float64)
    nb = U.shape[1] // B
    Rs = np.empty((nb, B, B))
    ns = np.empty(nb, dtype=np.int32)
    for b in range(nb):
        Rs[b], ns[b], _ = greedy_rotation(U[:, b * B:(b + 1) * B], Qs)
    return Rs, ns


def rotate_dense(X_bf16, d, Rs):
    """V = (X diag(d)) BlockDiag(R_1 .. R_nb) as float64 (G_t of Eq. 10 with dense blocks)."""
    U = bf16_to_f64(_c(X_bf16, np.uint16))
    if d is not None:
        U = U * np.asarray(d, dtype=np.float32).astype(np.float64)
    Rs = np.asarray(Rs, dtype=np.float64)
    B = Rs.shape[1]
    V = np.empty_like(U)
    for b in range(Rs.shape[0]):
        V[:, b * B:(b + 1) * B] = U[:, b * B:(b + 1) * B] @ Rs[b]
    return V


def rotate_weights_dense(W, d, Rs):
    """W' = BlockDiag(R_b)^T diag(1/d) W as float64 (H_t of Eq. 10 with dense blocks)."""
    Wd = np.asarray(W, dtype=np.float32).astype(np.float64)
    if d is not None:
        Wd = Wd / np.asarray(d, dtype=np.float32).astype(np.float64)[:, None]
    Rs = np.asarray(Rs, dtype=np.float64)
    B = Rs.shape[1]
    out = np.empty_like(Wd)
    for b in range(Rs.shape[0]):
        out[b * B:(b + 1) * B] = Rs[b].T @ Wd[b * B:(b + 1) * B]
    return out


def linear_dense(X_bf16, W, d, Rs, bias=None, wbits=8, exact_blas=False):
    """Whole path with dense rotation blocks (float32 values of Rs, as the library takes them)."""
    Rs = np.asarray(Rs, dtype=np.float32)
    B = Rs.shape[1]
    Xq, sx = quant_tokens(rotate_dense(X_bf16, d, Rs))
    Wq, sw = quant_weights(rotate_weights_dense(W, d, Rs), wbits, B)
    group = B if wbits == 4 else None
    acc = (acc_exact_blas if exact_blas else igemm)(Xq, Wq, group)
    Y, Yd = dequant(acc, sx, sw, bias, return_f64=True)
    return dict(Xq=Xq, sx=sx, Wq=Wq, sw=sw, acc=acc, Y=Y, Yd=Yd)


def rotate_dense_rpr(X_bf16, d, R1s, perm, R2s):
    """V = (X diag(d)) BlockDiag(R1) P BlockDiag(R2) as float64: G_t of Eq. 10 in full, with dense
    blocks for both rotations; (U P)[k'] = U[perm[k']]."""
    V1 = rotate_dense(X_bf16, d, R1s)
    V2 = V1[:, np.asarray(perm, dtype=np.int64)]
    R2s = np.asarray(R2s, dtype=np.float64)
    B = R2s.shape[1]
    out = np.empty_like(V2)
    for b in range(R2s.shape[0]):
        out[:, b * B:(b + 1) * B] = V2[:, b * B:(b + 1) * B] @ R2s[b]
    return out


def rotate_weights_dense_rpr(W, d, R1s, perm, R2s):
    """W' = BlockDiag(R2)^T P^T BlockDiag(R1)^T diag(1/d) W as float64 (H_t of Eq. 10 in full)."""
    W1 = rotate_weights_dense(W, d, R1s)
    W2 = W1[np.asarray(perm, dtype=np.int64)]                 # (P^T W1)[k'] = W1[perm[k']]
    R2s = np.asarray(R2s, dtype=np.float64)
    B = R2s.shape[1]
    out = np.empty_like(W2)
    for b in range(R2s.shape[0]):
        out[b * B:(b + 1) * B] = R2s[b].T @ W2[b * B:(b + 1) * B]
    return out


def linear_dense_rpr(X_bf16, W, d, R1s, perm, R2s, bias=None, wbits=8, exact_blas=False):
    R1s = np.asarray(R1s, dtype=np.float32)
    R2s = np.asarray(R2s, dtype=np.float32)
    B = R1s.shape[1]
    Xq, sx = quant_tokens(rotate_dense_rpr(X_bf16, d, R1s, perm, R2s))
    Wq, sw = quant_weights(rotate_weights_dense_rpr(W, d, R1s, perm, R2s), wbits, B)
    group = B if wbits == 4 else None
    acc = (acc_exact_blas if exact_blas else igemm)(Xq, Wq, group)
    Y, Yd = dequant(acc, sx, sw, bias, return_f64=True)
    return dict(Xq=Xq, sx=sx, Wq=Wq, sw=sw, acc=acc, Y=Y, Yd=Yd)


def calibrate_time_rotation(X_bf16, d, Qs1, Qs2, B=128):
    """The per-group calibration of Sec. 3.2 end to end on calibration activations X (times d):
    greedy first rotation (Eq. 6-7), zigzag permutation from the per-channel maxima after it, greedy
    second rotation on the rotated, permuted activations.  Returns (R1s, n1, perm, R2s, n2)."""
    R1s, n1 = greedy_rotations(X_bf16, d, Qs1, B)
    R1s32 = R1s.astype(np.float32)
    V1 = rotate_dense(X_bf16, d, R1s32)
    perm = zigzag(np.abs(V1).max(axis=0), B)
    V2 = V1[:, perm.astype(np.int64)]
    nb = V2.shape[1] // B
    R2s = np.empty((nb, B, B))
    n2 = np.empty(nb, dtype=np.int32)
    for b in range(nb):
        R2s[b], n2[b], _ = greedy_rotation(V2[:, b * B:(b + 1) * B], Qs2)
    return R1s32, n1, perm, R2s.astype(np.float32), n2


# ---- attention sharing (Sec. 3.3) ------------------------------------------------------------

def cosine_similarity(A_bf16, B_bf16):
    """Eq. 11 per row: cos(A, B) = A.B / (|A| |B|) for bf16 inputs [n, L], in float64.
    A row where either vector is all zero has no direction: 0."""
    A = bf16_to_f64(np.atleast_2d(A_bf16))
    Bm = bf16_to_f64(np.atleast_2d(B_bf16))
    out = np.zeros(A.shape[0], dtype=np.float64)
    for i in range(A.shape[0]):
        dot = float(np.dot(A[i], Bm[i]))
        na = float(np.dot(A[i], A[i]))
        nbb = float(np.dot(Bm[i], Bm[i]))
        if na > 0.0 and nbb > 0.0:
            out[i] = dot / (np.sqrt(na) * np.sqrt(nbb))
    return out


def share_plan(sim, threshold):
    """Which transformer blocks share attention between the conditional and the unconditional
    pass (Sec. 3.3: the blocks whose attention outputs are similar at every time step):
    sim [n_steps, n_blocks] of Eq. 11 values -> 0/1 per block, 1 where min over the steps >= threshold."""
    sim = np.asarray(sim, dtype=np.float64)
    return (sim.min(axis=0) >= threshold).astype(np.int32)


def channel_absmax(X_bf16, d=None, rotate_first=False, B=128):
    """max over tokens of |(X diag(d))[i, k]|, or of |((X diag(d)) R)[i, k]| when rotate_first."""
    if rotate_first:
        V = rotate(X_bf16, d, B)
    else:
        V = bf16_to_f64(X_bf16)
        if d is not None:
            V = V * np.asarray(d, dtype=np.float64)[None, :]
    return np.abs(V).max(axis=0) if V.shape[0] else np.zeros(V.shape[1])


def weight_row_absmax(W):
    return np.abs(np.asarray(W, dtype=np.float64)).max(axis=1)


def smooth_diag(xmax, wmax, alpha):
    """Eq. 5, Delta_j = max|X_j|^alpha / max|W_j|^(1-alpha), returned as the multiplier of the
    activations d_j = 1 / Delta_j (Eq. 9/10 multiply X by the diagonal where Eq. 4 divides by it).
    A channel whose activation or weight maximum is zero keeps d_j = 1."""
    xmax = np.asarray(xmax, dtype=np.float64)
    wmax = np.asarray(wmax, dtype=np.float64)
    d = np.ones_like(xmax)
    ok = (xmax > 0) & (wmax > 0)
    d[ok] = wmax[ok] ** (1.0 - alpha) / xmax[ok] ** alpha
    return d


def pack_int4(Wq):
    Wq = _c(Wq, np.int8)
    K, N = Wq.shape
    out = np.empty((K // 2, N), dtype=np.uint8)
    _chk(lib().trdq_oracle_pack_int4(_ptr(Wq), K, N, _ptr(out)), "pack_int4")
    return out


def unpack_int4(packed):
    packed = _c(packed, np.uint8)
    K2, N = packed.shape
    out = np.empty((K2 * 2, N), dtype=np.int8)
    _chk(lib().trdq_oracle_unpack_int4(_ptr(packed), K2 * 2, N, _ptr(out)), "unpack_int4")
    return out


def igemm(Xq, Wq, group=None):
    """int32 accumulators: [M, N] when group is None, else [K/group, M, N]."""
    Xq, Wq = _c(Xq, np.int8), _c(Wq, np.int8)
    M, K = Xq.shape
    K2, N = Wq.shape
    assert K == K2
    g = K if group is None else group
    ng = K // g
    acc = np.empty((ng, M, N), dtype=np.int32)
    _chk(lib().trdq_oracle_igemm(_ptr(Xq), _ptr(Wq), M, K, N, g, _ptr(acc)), "igemm")
    return acc[0] if group is None else acc


def acc_exact_blas(Xq, Wq, group=None):
    """Same integer sums as igemm through a float64 library matmul.

    |partial sums| <= 127*127*K < 2^53, so every float64 operation is exact and the
    result equals the int32 loop bit for bit (pinned in the tests on small shapes)."""
    Xq, Wq = np.asarray(Xq), np.asarray(Wq)
    M, K = Xq.shape
    g = K if group is None else group
    ng = K // g
    Xd, Wd = Xq.astype(np.float64), Wq.astype(np.float64)
    out = np.empty((ng, M, Wq.shape[1]), dtype=np.int32)
    for b in range(ng):
        out[b] = (Xd[:, b * g:(b + 1) * g] @ Wd[b * g:(b + 1) * g]).astype(np.int32)
    return out[0] if group is None else out


def dequant(acc, sx, sw, bias=None, return_f64=False):
    acc = _c(acc, np.int32)
    if acc.ndim == 2:
        ng, (M, N) = 1, acc.shape
    else:
        ng, M, N = acc.shape
    sx = _c(sx, np.float64)
    sw = _c(sw, np.float64)
    bias = _c(bias, np.float32)
    Y = np.empty((M, N), dtype=np.uint16)
    Yd = np.empty((M, N), dtype=np.float64) if return_f64 else None
    _chk(lib().trdq_oracle_dequant(_ptr(acc), _ptr(sx), _ptr(sw), _ptr(bias), M, N, ng,
                                   _ptr(Y), _ptr(Yd)), "dequant")
    return (Y, Yd) if return_f64 else Y


def linear(X_bf16, W, d=None, bias=None, B=128, wbits=8, exact_blas=False, abits=8):
    """Whole path; returns a dict with Xq, sx, Wq, sw, acc, Y (bf16 bits) and Yd (float64).

    exact_blas=True replaces only the integer-product step by acc_exact_blas."""
    Xq, sx = rotate_quant(X_bf16, d, B, abits)
    Wq, sw = prepare_weights(W, d, B, wbits)
    group = B if wbits == 4 else None
    acc = (acc_exact_blas if exact_blas else igemm)(Xq, Wq, group)
    Y, Yd = dequant(acc, sx, sw, bias, return_f64=True)
    return dict(Xq=Xq, sx=sx, Wq=Wq, sw=sw, acc=acc, Y=Y, Yd=Yd)


def linear_c(X_bf16, W, d=None, bias=None, B=128, wbits=8):
    """The single C entry point running every step (used for timing the baseline)."""
    X = _c(X_bf16, np.uint16)
    W = _c(W, np.float32)
    M, K = X.shape
    N = W.shape[1]
    d = _c(d, np.float32)
    bias = _c(bias, np.float32)
    Y = np.empty((M, N), dtype=np.uint16)
    _chk(lib().trdq_oracle_linear(_ptr(X), M, K, K, _ptr(W), N, _ptr(d), _ptr(bias), B, wbits,
                                  None, None, None, None, None, _ptr(Y)), "linear")
    return Y
