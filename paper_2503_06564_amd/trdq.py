"""ctypes binding of libtrdq.so: same names as the C ABI (include/trdq.h), marshalling only.

Every step of the path runs in the library's HIP kernels; torch appears only as the owner
of device memory and streams (tensor.data_ptr(), torch.cuda.current_stream()).  The library
is loaded on first use and a missing build raises: there is no CPU fallback.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtrdq.so")

OK, ERR_NULL, ERR_SHAPE, ERR_RANGE, ERR_UNSUPPORTED, ERR_MISMATCH, ERR_ALLOC, ERR_HIP = range(8)
BLOCK = 128

SYMBOLS = [
    "trdq_status_str", "trdq_abi_version",
    "trdq_table_create", "trdq_table_lookup", "trdq_table_sizes", "trdq_table_destroy",
    "trdq_prepare_weights", "trdq_weights_info", "trdq_weights_export",
    "trdq_weights_export_packed", "trdq_weights_nbytes", "trdq_weights_destroy",
    "trdq_rotate_quant", "trdq_rotate_quant_warm", "trdq_qgemm", "trdq_linear_fused", "trdq_linear_fused_asym",
    "trdq_layer_create", "trdq_layer_set_group", "trdq_layer_forward", "trdq_layer_weights",
    "trdq_layer_destroy", "trdq_qgemm_set_variant", "trdq_qgemm_num_variants",
    "trdq_zigzag_permutation", "trdq_prepare_weights_rpr", "trdq_rotate_quant_rpr",
    "trdq_channel_absmax", "trdq_weight_row_absmax", "trdq_smooth_diag",
    "trdq_rotate_quant_asym", "trdq_qgemm_asym", "trdq_rotate_quant_bits",
    "trdq_cosine_similarity", "trdq_cosine_similarity_static", "trdq_share_plan",
    "trdq_rotation_create", "trdq_rotation_destroy", "trdq_prepare_weights_dense", "trdq_rotate_quant_dense",
    "trdq_greedy_rotation", "trdq_prepare_weights_dense_rpr", "trdq_rotate_quant_dense_rpr",
    "trdq_rotate_quant_dense_rpr_ws", "trdq_rotate_quant_dense_rpr_ws_nbytes",
    "trdq_channel_absmax_dense", "trdq_greedy_rotation_second",
    "trdq_peak_mfma_i8", "trdq_peak_mfma_i8_data", "trdq_peak_stream",
    "trdq_xq_tiled_nbytes", "trdq_rotate_quant_tiled", "trdq_xq_untile", "trdq_qgemm_tiled_supported", "trdq_qgemm_tiled_preferred",
    "trdq_qgemm_tiled",
    "trdq_rotate_quant_rpr_asym", "trdq_prepare_weights_asym", "trdq_weights_export_zero_points", "trdq_qgemm_asym_weights",
]

_lib = None


class TrdqError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_str(status)} (status {status})")


def lib():
    """The loaded library; raises if libtrdq.so has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2503_06564_amd.build` "
                "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        i32, i64, p = C.c_int, C.c_int64, C.c_void_p
        L.trdq_status_str.restype = C.c_char_p
        L.trdq_status_str.argtypes = [i32]
        L.trdq_abi_version.restype = i32
        L.trdq_table_create.argtypes = [i32, i32, p, C.POINTER(p)]
        L.trdq_table_lookup.argtypes = [p, i32, C.POINTER(i32)]
        L.trdq_table_sizes.argtypes = [p, C.POINTER(i32), C.POINTER(i32)]
        L.trdq_table_destroy.argtypes = [p]
        L.trdq_table_destroy.restype = None
        L.trdq_prepare_weights.argtypes = [p, i32, i32, p, i32, i32, p, C.POINTER(p)]
        L.trdq_weights_info.argtypes = [p, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
        L.trdq_weights_export.argtypes = [p, p, p]
        L.trdq_weights_export_packed.argtypes = [p, p]
        L.trdq_weights_nbytes.argtypes = [p, C.POINTER(i64)]
        L.trdq_weights_destroy.argtypes = [p]
        L.trdq_weights_destroy.restype = None
        L.trdq_rotate_quant.argtypes = [p, i64, i32, i64, p, i32, p, p, p]
        L.trdq_rotate_quant_warm.argtypes = [p, i64, i32, i64, p, i32, p, p, p, p]
        L.trdq_qgemm.argtypes = [p, p, p, i64, p, p, i64, p, p]
        L.trdq_linear_fused.argtypes = [p, i64, i64, p, p, p, p, i64, p]
        L.trdq_linear_fused_asym.argtypes = [p, i64, i64, p, p, p, p, i64, p]
        L.trdq_layer_create.argtypes = [p, i32, i32, i32, C.POINTER(p)]
        L.trdq_layer_set_group.argtypes = [p, i32, p, p, p]
        L.trdq_layer_forward.argtypes = [p, i32, p, i64, p, p, i32, p, p, p]
        L.trdq_layer_weights.argtypes = [p, i32, C.POINTER(p)]
        L.trdq_layer_destroy.argtypes = [p]
        L.trdq_layer_destroy.restype = None
        L.trdq_qgemm_set_variant.argtypes = [i32]
        L.trdq_zigzag_permutation.argtypes = [p, i32, i32, p]
        L.trdq_rotate_quant_asym.argtypes = [p, i64, i32, i64, p, i32, p, p, p, p, p]
        L.trdq_rotate_quant_bits.argtypes = [p, i64, i32, i64, p, i32, i32, p, p, p, p]
        L.trdq_cosine_similarity.argtypes = [p, p, i32, i64, i64, i64, p, p, p]
        L.trdq_cosine_similarity_static.argtypes = [p, p, i32, i64, i64, i64, p, p]
        L.trdq_xq_tiled_nbytes.argtypes = [i64, i32]
        L.trdq_xq_tiled_nbytes.restype = i64
        L.trdq_rotate_quant_tiled.argtypes = [p, i64, i32, i64, p, i32, p, p, p, p]
        L.trdq_xq_untile.argtypes = [p, i64, i32, p, p]
        L.trdq_qgemm_tiled_supported.argtypes = [p, i64]
        L.trdq_qgemm_tiled_preferred.argtypes = [p, i64]
        L.trdq_qgemm_tiled.argtypes = [p, p, p, i64, p, p, i64, p, p]
        L.trdq_rotate_quant_rpr_asym.argtypes = [p, i64, i32, i64, p, p, i32, p, p, p, p, p]
        L.trdq_prepare_weights_asym.argtypes = [p, i32, i32, p, i32, i32, p, C.POINTER(p)]
        L.trdq_weights_export_zero_points.argtypes = [p, p]
        L.trdq_qgemm_asym_weights.argtypes = [p, p, p, p, p, i64, p, p, i64, p, p]
        L.trdq_share_plan.argtypes = [p, i32, i32, C.c_float, p]
        L.trdq_peak_mfma_i8.argtypes = [p, i32, i32, i32, C.POINTER(C.c_int64), p]
        L.trdq_peak_mfma_i8_data.argtypes = [p, i32, i32, i32, C.POINTER(C.c_int64), p]
        L.trdq_peak_stream.argtypes = [p, p, i64, p]
        L.trdq_rotation_create.argtypes = [p, p, i32, i32, p, C.POINTER(p)]
        L.trdq_rotation_destroy.argtypes = [p]
        L.trdq_rotation_destroy.restype = None
        L.trdq_prepare_weights_dense.argtypes = [p, i32, i32, p, i32, p, C.POINTER(p)]
        L.trdq_rotate_quant_dense.argtypes = [p, i64, i64, p, p, p, p]
        L.trdq_greedy_rotation.argtypes = [p, i64, i32, i64, p, i32, p, i32, p, p, p]
        L.trdq_prepare_weights_dense_rpr.argtypes = [p, i32, i32, p, p, p, i32, p, C.POINTER(p)]
        L.trdq_rotate_quant_dense_rpr.argtypes = [p, i64, i64, p, p, p, p, p, p]
        L.trdq_rotate_quant_dense_rpr_ws.argtypes = [p, i64, i64, p, p, p, p, p, p, C.c_size_t, p]
        L.trdq_rotate_quant_dense_rpr_ws_nbytes.argtypes = [i64, i32]
        L.trdq_rotate_quant_dense_rpr_ws_nbytes.restype = C.c_size_t
        L.trdq_channel_absmax_dense.argtypes = [p, i64, i64, p, p, p]
        L.trdq_greedy_rotation_second.argtypes = [p, i64, i64, p, p, p, i32, p, p, p]
        L.trdq_qgemm_asym.argtypes = [p, p, p, p, i64, p, p, i64, p, p]
        L.trdq_channel_absmax.argtypes = [p, i64, i32, i64, p, i32, i32, p, p]
        L.trdq_weight_row_absmax.argtypes = [p, i32, i32, p, p]
        L.trdq_smooth_diag.argtypes = [p, p, i32, C.c_float, p, p]
        L.trdq_prepare_weights_rpr.argtypes = [p, i32, i32, p, p, i32, i32, p, C.POINTER(p)]
        L.trdq_rotate_quant_rpr.argtypes = [p, i64, i32, i64, p, p, i32, p, p, p, p]
        L.trdq_qgemm_num_variants.restype = i32
        _lib = L
    return _lib


def status_str(status):
    return lib().trdq_status_str(int(status)).decode()


def _check(status, where):
    if status != OK:
        raise TrdqError(status, where)


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return t.ctypes.data


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


# ------------------------------------------------------------------ table

class Table:
    def __init__(self, n_steps, n_groups, mapping=None):
        import numpy as np
        h = C.c_void_p()
        m = None if mapping is None else np.ascontiguousarray(mapping, dtype=np.int32)
        _check(lib().trdq_table_create(n_steps, n_groups, _ptr(m), C.byref(h)), "trdq_table_create")
        self.handle = h

    def lookup(self, step):
        g = C.c_int()
        _check(lib().trdq_table_lookup(self.handle, step, C.byref(g)), "trdq_table_lookup")
        return g.value

    def sizes(self):
        a, b = C.c_int(), C.c_int()
        _check(lib().trdq_table_sizes(self.handle, C.byref(a), C.byref(b)), "trdq_table_sizes")
        return a.value, b.value

    def close(self):
        if self.handle:
            lib().trdq_table_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---------------------------------------------------------------- weights

class Weights:
    """Handle returned by trdq_prepare_weights (or borrowed from a Layer)."""

    def __init__(self, handle, owned=True):
        self.handle = handle
        self.owned = owned

    def info(self):
        k, n, b = C.c_int(), C.c_int(), C.c_int()
        _check(lib().trdq_weights_info(self.handle, C.byref(k), C.byref(n), C.byref(b)), "trdq_weights_info")
        return k.value, n.value, b.value

    def nbytes(self):
        v = C.c_int64()
        _check(lib().trdq_weights_nbytes(self.handle, C.byref(v)), "trdq_weights_nbytes")
        return v.value

    def export(self):
        """(codes int8 [K, N], scales float32 [N] or [K/128, N]) as numpy arrays."""
        import numpy as np
        K, N, wbits = self.info()
        codes = np.empty((K, N), dtype=np.int8)
        scales = np.empty((K // BLOCK, N) if wbits == 4 else (N,), dtype=np.float32)
        _check(lib().trdq_weights_export(self.handle, _ptr(codes), _ptr(scales)), "trdq_weights_export")
        return codes, scales

    def export_packed(self):
        import numpy as np
        K, N, _ = self.info()
        out = np.empty((K // 2, N), dtype=np.uint8)
        _check(lib().trdq_weights_export_packed(self.handle, _ptr(out)), "trdq_weights_export_packed")
        return out

    def close(self):
        if self.handle and self.owned:
            lib().trdq_weights_destroy(self.handle)
        self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def prepare_weights(W, diag=None, block=BLOCK, wbits=8, stream=None):
    """W: float32 device tensor [K, N]; diag: float32 device tensor [K] or None."""
    K, N = W.shape
    h = C.c_void_p()
    _check(lib().trdq_prepare_weights(_ptr(W), K, N, _ptr(diag), block, wbits, _stream(stream), C.byref(h)),
           "trdq_prepare_weights")
    return Weights(h)


def channel_absmax(X, diag, mag, rotate=False, block=BLOCK, stream=None):
    """mag[k] = max_i |(X diag)[i, k]|, or of the once-rotated activations when rotate is set."""
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    _check(lib().trdq_channel_absmax(_ptr(X), M, K, ldx, _ptr(diag), int(bool(rotate)), block, _ptr(mag),
                                     _stream(stream)), "trdq_channel_absmax")


def weight_row_absmax(W, wmax, stream=None):
    K, N = W.shape
    _check(lib().trdq_weight_row_absmax(_ptr(W), K, N, _ptr(wmax), _stream(stream)), "trdq_weight_row_absmax")


def smooth_diag(xmax, wmax, alpha, diag, stream=None):
    """Eq. 5 as the multiplier of the activations: diag = wmax^(1-alpha) / xmax^alpha."""
    _check(lib().trdq_smooth_diag(_ptr(xmax), _ptr(wmax), xmax.shape[0], float(alpha), _ptr(diag), _stream(stream)),
           "trdq_smooth_diag")


def zigzag_permutation(chan_mag, block=BLOCK):
    """chan_mag: host float32 array [K] of per-channel magnitudes -> host int32 array perm[K]."""
    import numpy as np
    mag = np.ascontiguousarray(chan_mag, dtype=np.float32)
    perm = np.empty(mag.shape[0], dtype=np.int32)
    _check(lib().trdq_zigzag_permutation(_ptr(mag), mag.shape[0], block, _ptr(perm)), "trdq_zigzag_permutation")
    return perm


def prepare_weights_rpr(W, diag, perm, block=BLOCK, wbits=8, stream=None):
    """Full H_t(W) of Eq. 9; perm: int32 device tensor [K]."""
    K, N = W.shape
    h = C.c_void_p()
    _check(lib().trdq_prepare_weights_rpr(_ptr(W), K, N, _ptr(diag), _ptr(perm), block, wbits, _stream(stream),
                                          C.byref(h)), "trdq_prepare_weights_rpr")
    return Weights(h)


# ----------------------------------------------------------------- online

def rotate_quant_rpr(X, diag, perm, Xq, sx, block=BLOCK, stream=None, warm=None):
    """Full G_t(X) of Eq. 9 and the per-token quantiser; perm: int32 device tensor [K]."""
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    _check(lib().trdq_rotate_quant_rpr(_ptr(X), M, K, ldx, _ptr(diag), _ptr(perm), block, _ptr(Xq), _ptr(sx),
                                       warm.handle if warm is not None else None, _stream(stream)),
           "trdq_rotate_quant_rpr")


def rotate_quant(X, diag, Xq, sx, block=BLOCK, stream=None, warm=None):
    """X: bf16 [M, K] (row stride X.stride(0)); Xq: int8 [M, K]; sx: float32 [M].
    warm: the Weights of the product that follows (their codes are read once on the way)."""
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    if warm is None:
        _check(lib().trdq_rotate_quant(_ptr(X), M, K, ldx, _ptr(diag), block, _ptr(Xq), _ptr(sx), _stream(stream)),
               "trdq_rotate_quant")
    else:
        _check(lib().trdq_rotate_quant_warm(_ptr(X), M, K, ldx, _ptr(diag), block, _ptr(Xq), _ptr(sx), warm.handle,
                                            _stream(stream)), "trdq_rotate_quant_warm")


class Rotation:
    """Dense rotation blocks R (float32 [K/128, 128, 128] on the device) with an optional diagonal."""

    def __init__(self, R, diag=None, stream=None):
        self.K = R.shape[0] * BLOCK
        h = C.c_void_p()
        _check(lib().trdq_rotation_create(_ptr(R), _ptr(diag), self.K, BLOCK, _stream(stream), C.byref(h)),
               "trdq_rotation_create")
        self.handle = h

    def close(self):
        if self.handle:
            lib().trdq_rotation_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def greedy_rotation(X, diag, Q, R_out, block=BLOCK, stream=None):
    """Eq. 6-7 per block: X bf16 [M, K], Q float64 [n_steps, 128, 128], R_out float32 [K/128, 128, 128] (written).
    Returns the chosen step counts as a numpy int32 array [K/128]."""
    import numpy as np
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    n = np.zeros(K // block, dtype=np.int32)
    _check(lib().trdq_greedy_rotation(_ptr(X), M, K, ldx, _ptr(diag), block, _ptr(Q), Q.shape[0], _ptr(R_out),
                                      n.ctypes.data, _stream(stream)), "trdq_greedy_rotation")
    return n


def channel_absmax_dense(X, rot, mag, stream=None):
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    _check(lib().trdq_channel_absmax_dense(_ptr(X), M, ldx, rot.handle, _ptr(mag), _stream(stream)),
           "trdq_channel_absmax_dense")


def greedy_rotation_second(X, rot1, perm, Q, R_out, stream=None):
    """Eq. 6-7 for the second rotation: the search runs on ((X d) R1)[:, perm]."""
    import numpy as np
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    n = np.zeros(K // BLOCK, dtype=np.int32)
    _check(lib().trdq_greedy_rotation_second(_ptr(X), M, ldx, rot1.handle, _ptr(perm), _ptr(Q), Q.shape[0], _ptr(R_out),
                                             n.ctypes.data, _stream(stream)), "trdq_greedy_rotation_second")
    return n


def prepare_weights_dense(W, rot, wbits=8, stream=None):
    K, N = W.shape
    h = C.c_void_p()
    _check(lib().trdq_prepare_weights_dense(_ptr(W), K, N, rot.handle, wbits, _stream(stream), C.byref(h)),
           "trdq_prepare_weights_dense")
    return Weights(h)


def rotate_quant_dense(X, rot, Xq, sx, stream=None):
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    _check(lib().trdq_rotate_quant_dense(_ptr(X), M, ldx, rot.handle, _ptr(Xq), _ptr(sx), _stream(stream)),
           "trdq_rotate_quant_dense")


def prepare_weights_dense_rpr(W, rot1, perm, rot2, wbits=8, stream=None):
    K, N = W.shape
    h = C.c_void_p()
    _check(lib().trdq_prepare_weights_dense_rpr(_ptr(W), K, N, rot1.handle, _ptr(perm), rot2.handle, wbits,
                                                _stream(stream), C.byref(h)), "trdq_prepare_weights_dense_rpr")
    return Weights(h)


def rotate_quant_dense_rpr(X, rot1, perm, rot2, Xq, sx, stream=None):
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    _check(lib().trdq_rotate_quant_dense_rpr(_ptr(X), M, ldx, rot1.handle, _ptr(perm), rot2.handle, _ptr(Xq), _ptr(sx),
                                             _stream(stream)), "trdq_rotate_quant_dense_rpr")


def rotate_quant_dense_rpr_ws_nbytes(M, K):
    """bytes of device workspace rotate_quant_dense_rpr_ws needs (0 up to K = 1536 below 16384 tokens)"""
    return int(lib().trdq_rotate_quant_dense_rpr_ws_nbytes(M, K))


def rotate_quant_dense_rpr_ws(X, rot1, perm, rot2, Xq, sx, ws, stream=None):
    """rotate_quant_dense_rpr with a device workspace `ws` (any dtype, contiguous; None where none is needed)"""
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(lib().trdq_rotate_quant_dense_rpr_ws(_ptr(X), M, ldx, rot1.handle, _ptr(perm), rot2.handle, _ptr(Xq), _ptr(sx),
                                                _ptr(ws), ws_bytes, _stream(stream)), "trdq_rotate_quant_dense_rpr_ws")


def bind_rotate_quant_dense(X, rot, Xq, sx, stream=None):
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    f = lib().trdq_rotate_quant_dense
    args = (C.c_void_p(_ptr(X)), C.c_int64(M), C.c_int64(ldx), rot.handle, C.c_void_p(_ptr(Xq)), C.c_void_p(_ptr(sx)),
            C.c_void_p(_stream(stream)))

    def call():
        st = f(*args)
        if st != OK:
            raise TrdqError(st, "trdq_rotate_quant_dense")
    return call


def cosine_similarity(A, B, acc_ws, out, stream=None):
    """Eq. 11 per row of A, B (bf16 [n_seg, L], rows may be strided); acc_ws float64 [3 * n_seg], out float32 [n_seg]."""
    n_seg, L = A.shape
    sa = A.stride(0) if n_seg > 1 else max(L, A.stride(0))
    sb = B.stride(0) if n_seg > 1 else max(L, B.stride(0))
    _check(lib().trdq_cosine_similarity(_ptr(A), _ptr(B), n_seg, L, sa, sb, _ptr(acc_ws), _ptr(out), _stream(stream)),
           "trdq_cosine_similarity")


COSINE_STATIC_MAX_SEG = 4096


def cosine_similarity_static(A, B, out, stream=None):
    """cosine_similarity without a workspace: the accumulators are a fixed array inside the library
    (at most COSINE_STATIC_MAX_SEG segments; calls that overlap on one GPU race)."""
    n_seg, L = A.shape
    sa = A.stride(0) if n_seg > 1 else max(L, A.stride(0))
    sb = B.stride(0) if n_seg > 1 else max(L, B.stride(0))
    _check(lib().trdq_cosine_similarity_static(_ptr(A), _ptr(B), n_seg, L, sa, sb, _ptr(out), _stream(stream)),
           "trdq_cosine_similarity_static")


def peak_mfma_i8(sink, workgroups, waves, iters, stream=None, random_data=False):
    """Yardstick: iters x 8 register-only int8 matrix instructions per wave, on operands of ones or of
    pseudo-random bytes; returns the launch's operation count."""
    ops = C.c_int64(0)
    f = lib().trdq_peak_mfma_i8_data if random_data else lib().trdq_peak_mfma_i8
    _check(f(_ptr(sink), workgroups, waves, iters, C.byref(ops), _stream(stream)),
           "trdq_peak_mfma_i8_data" if random_data else "trdq_peak_mfma_i8")
    return ops.value


def peak_stream(src, dst, stream=None):
    """Yardstick: dst (int8) <- low byte of every 16-bit element of src; 2 bytes read, 1 written per element."""
    _check(lib().trdq_peak_stream(_ptr(src), _ptr(dst), src.numel(), _stream(stream)), "trdq_peak_stream")


def share_plan(sim, threshold):
    """sim: float32 numpy [n_steps, n_blocks] -> int32 [n_blocks] (1 = share attention)."""
    import numpy as np
    sim = np.ascontiguousarray(sim, dtype=np.float32)
    out = np.empty(sim.shape[1], dtype=np.int32)
    _check(lib().trdq_share_plan(sim.ctypes.data, sim.shape[0], sim.shape[1], float(threshold), out.ctypes.data),
           "trdq_share_plan")
    return out


def rotate_quant_bits(X, diag, Xq, sx, abits, block=BLOCK, stream=None, warm=None):
    """Symmetric per-token codes of `abits` bits (2..8), one per int8."""
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    _check(lib().trdq_rotate_quant_bits(_ptr(X), M, K, ldx, _ptr(diag), block, abits, _ptr(Xq), _ptr(sx),
                                        warm.handle if warm is not None else None, _stream(stream)),
           "trdq_rotate_quant_bits")


def rotate_quant_asym(X, diag, Xq, sx, zc, block=BLOCK, stream=None, warm=None):
    """Asymmetric per-token quantiser (Eq. 1-3): Xq int8 [M, K] holds q - 128, zc int32 [M] holds 128 - z."""
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    _check(lib().trdq_rotate_quant_asym(_ptr(X), M, K, ldx, _ptr(diag), block, _ptr(Xq), _ptr(sx), _ptr(zc),
                                        warm.handle if warm is not None else None, _stream(stream)),
           "trdq_rotate_quant_asym")


def qgemm_asym(w, Xq, sx, zc, Y, bias=None, acc_debug=None, stream=None):
    M = Xq.shape[0]
    ldy = Y.stride(0) if M > 1 else max(Y.shape[1], Y.stride(0))
    _check(lib().trdq_qgemm_asym(w.handle, _ptr(Xq), _ptr(sx), _ptr(zc), M, _ptr(bias), _ptr(Y), ldy,
                                 _ptr(acc_debug), _stream(stream)), "trdq_qgemm_asym")


def rotate_quant_rpr_asym(X, diag, perm, Xq, sx, zc, block=BLOCK, stream=None, warm=None):
    """rotate_quant_rpr with asymmetric codes (q - 128 in Xq, 128 - z in zc)."""
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    _check(lib().trdq_rotate_quant_rpr_asym(_ptr(X), M, K, ldx, _ptr(diag), _ptr(perm), block, _ptr(Xq), _ptr(sx),
                                            _ptr(zc), warm.handle if warm is not None else None, _stream(stream)),
           "trdq_rotate_quant_rpr_asym")


def prepare_weights_asym(W, diag, block=BLOCK, wbits=8, stream=None):
    """Weights with a zero point per output channel (Eq. 1-3 on H_t(W)); int8 storage of q - 128."""
    K, N = W.shape
    h = C.c_void_p()
    _check(lib().trdq_prepare_weights_asym(_ptr(W), K, N, _ptr(diag), block, wbits, _stream(stream), C.byref(h)),
           "trdq_prepare_weights_asym")
    return Weights(h)


def weights_zero_points(w):
    """z_w int32 [N] (host) of an asymmetric weight set."""
    import numpy as np
    K, N, _ = w.info()
    z = np.empty(N, dtype=np.int32)
    _check(lib().trdq_weights_export_zero_points(w.handle, _ptr(z)), "trdq_weights_export_zero_points")
    return z


def qgemm_asym_weights(w, Xq, sx, zc, rowsum_ws, Y, bias=None, acc_debug=None, stream=None):
    """Product against asymmetric weights; zc None for symmetric activation codes; rowsum_ws int32 [M] workspace."""
    M = Xq.shape[0]
    ldy = Y.stride(0) if M > 1 else max(Y.shape[1], Y.stride(0))
    _check(lib().trdq_qgemm_asym_weights(w.handle, _ptr(Xq), _ptr(sx), _ptr(zc), _ptr(rowsum_ws), M, _ptr(bias),
                                         _ptr(Y), ldy, _ptr(acc_debug), _stream(stream)), "trdq_qgemm_asym_weights")


def qgemm(w, Xq, sx, Y, bias=None, acc_debug=None, stream=None):
    M = Xq.shape[0]
    ldy = Y.stride(0) if M > 1 else max(Y.shape[1], Y.stride(0))
    _check(lib().trdq_qgemm(w.handle, _ptr(Xq), _ptr(sx), M, _ptr(bias), _ptr(Y), ldy, _ptr(acc_debug),
                            _stream(stream)), "trdq_qgemm")


# ---- the pair on block-tiled activation codes ---------------------------------------------------

def xq_tiled_nbytes(M, K):
    """Bytes of the block-tiled code buffer of an [M, K] activation matrix."""
    n = lib().trdq_xq_tiled_nbytes(M, K)
    if n < 0:
        raise TrdqError(ERR_SHAPE, "trdq_xq_tiled_nbytes")
    return n


def rotate_quant_tiled(X, diag, Xt, sx, block=BLOCK, stream=None, warm=None):
    """rotate_quant writing the codes in 1 KB blocks of 16 tokens x 64 channels; Xt: int8, xq_tiled_nbytes(M, K) bytes."""
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    _check(lib().trdq_rotate_quant_tiled(_ptr(X), M, K, ldx, _ptr(diag), block, _ptr(Xt), _ptr(sx),
                                         warm.handle if warm is not None else None, _stream(stream)),
           "trdq_rotate_quant_tiled")


def xq_untile(Xt, M, K, Xq, stream=None):
    """Xq int8 [M, K] dense <- the block-tiled codes Xt."""
    _check(lib().trdq_xq_untile(_ptr(Xt), M, K, _ptr(Xq), _stream(stream)), "trdq_xq_untile")


def qgemm_tiled_supported(w, M):
    return bool(lib().trdq_qgemm_tiled_supported(w.handle, M))


def qgemm_tiled_preferred(w, M):
    """True where the library itself (trdq_layer_forward) takes the tiled pair: supported and measured faster."""
    return bool(lib().trdq_qgemm_tiled_preferred(w.handle, M))


def qgemm_tiled(w, Xt, sx, Y, bias=None, acc_debug=None, stream=None):
    M = Y.shape[0]
    ldy = Y.stride(0) if M > 1 else max(Y.shape[1], Y.stride(0))
    _check(lib().trdq_qgemm_tiled(w.handle, _ptr(Xt), _ptr(sx), M, _ptr(bias), _ptr(Y), ldy, _ptr(acc_debug),
                                  _stream(stream)), "trdq_qgemm_tiled")


def bind_rotate_quant_tiled(X, diag, Xt, sx, block=BLOCK, stream=None, warm=None):
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    f = lib().trdq_rotate_quant_tiled
    args = (C.c_void_p(_ptr(X)), C.c_int64(M), C.c_int(K), C.c_int64(ldx), C.c_void_p(_ptr(diag)), C.c_int(block),
            C.c_void_p(_ptr(Xt)), C.c_void_p(_ptr(sx)), warm.handle if warm is not None else C.c_void_p(None),
            C.c_void_p(_stream(stream)))

    def call():
        st = f(*args)
        if st != OK:
            raise TrdqError(st, "trdq_rotate_quant_tiled")
    return call


def bind_qgemm_tiled(w, Xt, sx, Y, bias=None, acc_debug=None, stream=None):
    M = Y.shape[0]
    ldy = Y.stride(0) if M > 1 else max(Y.shape[1], Y.stride(0))
    f = lib().trdq_qgemm_tiled
    args = (w.handle, C.c_void_p(_ptr(Xt)), C.c_void_p(_ptr(sx)), C.c_int64(M), C.c_void_p(_ptr(bias)),
            C.c_void_p(_ptr(Y)), C.c_int64(ldy), C.c_void_p(_ptr(acc_debug)), C.c_void_p(_stream(stream)))

    def call():
        st = f(*args)
        if st != OK:
            raise TrdqError(st, "trdq_qgemm_tiled")
    return call


def linear_fused(X, diag, w, Y, bias=None, stream=None):
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    ldy = Y.stride(0) if M > 1 else max(Y.shape[1], Y.stride(0))
    _check(lib().trdq_linear_fused(_ptr(X), M, ldx, _ptr(diag), w.handle, _ptr(bias), _ptr(Y), ldy,
                                   _stream(stream)), "trdq_linear_fused")


def linear_fused_asym(X, diag, w, Y, bias=None, stream=None):
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    ldy = Y.stride(0) if M > 1 else max(Y.shape[1], Y.stride(0))
    _check(lib().trdq_linear_fused_asym(_ptr(X), M, ldx, _ptr(diag), w.handle, _ptr(bias), _ptr(Y), ldy,
                                        _stream(stream)), "trdq_linear_fused_asym")


# ---- pre-marshalled calls ---------------------------------------------------------------------
# For launch-bound loops: the arguments are converted to ctypes once; calling the returned
# function performs exactly one C call (same entry points, same semantics).

def bind_rotate_quant(X, diag, Xq, sx, block=BLOCK, stream=None, warm=None):
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    f = lib().trdq_rotate_quant_warm
    args = (C.c_void_p(_ptr(X)), C.c_int64(M), C.c_int(K), C.c_int64(ldx), C.c_void_p(_ptr(diag)), C.c_int(block),
            C.c_void_p(_ptr(Xq)), C.c_void_p(_ptr(sx)), warm.handle if warm is not None else C.c_void_p(None),
            C.c_void_p(_stream(stream)))

    def call():
        st = f(*args)
        if st != OK:
            raise TrdqError(st, "trdq_rotate_quant_warm")
    return call


def bind_rotate_quant_rpr(X, diag, perm, Xq, sx, block=BLOCK, stream=None, warm=None):
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    f = lib().trdq_rotate_quant_rpr
    args = (C.c_void_p(_ptr(X)), C.c_int64(M), C.c_int(K), C.c_int64(ldx), C.c_void_p(_ptr(diag)),
            C.c_void_p(_ptr(perm)), C.c_int(block), C.c_void_p(_ptr(Xq)), C.c_void_p(_ptr(sx)),
            warm.handle if warm is not None else C.c_void_p(None), C.c_void_p(_stream(stream)))

    def call():
        st = f(*args)
        if st != OK:
            raise TrdqError(st, "trdq_rotate_quant_rpr")
    return call


def bind_rotate_quant_asym(X, diag, Xq, sx, zc, block=BLOCK, stream=None, warm=None):
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    f = lib().trdq_rotate_quant_asym
    args = (C.c_void_p(_ptr(X)), C.c_int64(M), C.c_int(K), C.c_int64(ldx), C.c_void_p(_ptr(diag)), C.c_int(block),
            C.c_void_p(_ptr(Xq)), C.c_void_p(_ptr(sx)), C.c_void_p(_ptr(zc)),
            warm.handle if warm is not None else C.c_void_p(None), C.c_void_p(_stream(stream)))

    def call():
        st = f(*args)
        if st != OK:
            raise TrdqError(st, "trdq_rotate_quant_asym")
    return call


def bind_qgemm_asym(w, Xq, sx, zc, Y, bias=None, acc_debug=None, stream=None):
    M = Xq.shape[0]
    ldy = Y.stride(0) if M > 1 else max(Y.shape[1], Y.stride(0))
    f = lib().trdq_qgemm_asym
    args = (w.handle, C.c_void_p(_ptr(Xq)), C.c_void_p(_ptr(sx)), C.c_void_p(_ptr(zc)), C.c_int64(M),
            C.c_void_p(_ptr(bias)), C.c_void_p(_ptr(Y)), C.c_int64(ldy), C.c_void_p(_ptr(acc_debug)),
            C.c_void_p(_stream(stream)))

    def call():
        st = f(*args)
        if st != OK:
            raise TrdqError(st, "trdq_qgemm_asym")
    return call


def bind_qgemm(w, Xq, sx, Y, bias=None, acc_debug=None, stream=None):
    M = Xq.shape[0]
    ldy = Y.stride(0) if M > 1 else max(Y.shape[1], Y.stride(0))
    f = lib().trdq_qgemm
    args = (w.handle, C.c_void_p(_ptr(Xq)), C.c_void_p(_ptr(sx)), C.c_int64(M), C.c_void_p(_ptr(bias)),
            C.c_void_p(_ptr(Y)), C.c_int64(ldy), C.c_void_p(_ptr(acc_debug)), C.c_void_p(_stream(stream)))

    def call():
        st = f(*args)
        if st != OK:
            raise TrdqError(st, "trdq_qgemm")
    return call


def bind_linear_fused(X, diag, w, Y, bias=None, stream=None):
    M, K = X.shape
    ldx = X.stride(0) if M > 1 else max(K, X.stride(0))
    ldy = Y.stride(0) if M > 1 else max(Y.shape[1], Y.stride(0))
    f = lib().trdq_linear_fused
    args = (C.c_void_p(_ptr(X)), C.c_int64(M), C.c_int64(ldx), C.c_void_p(_ptr(diag)), w.handle,
            C.c_void_p(_ptr(bias)), C.c_void_p(_ptr(Y)), C.c_int64(ldy), C.c_void_p(_stream(stream)))

    def call():
        st = f(*args)
        if st != OK:
            raise TrdqError(st, "trdq_linear_fused")
    return call


def qgemm_set_variant(variant):
    _check(lib().trdq_qgemm_set_variant(variant), "trdq_qgemm_set_variant")


def qgemm_num_variants():
    return lib().trdq_qgemm_num_variants()


# ------------------------------------------------------------------ layer

class Layer:
    def __init__(self, table, K, N, wbits=8):
        h = C.c_void_p()
        _check(lib().trdq_layer_create(table.handle, K, N, wbits, C.byref(h)), "trdq_layer_create")
        self.handle = h
        self.K, self.N, self.wbits = K, N, wbits

    def set_group(self, g, diag, W, stream=None):
        _check(lib().trdq_layer_set_group(self.handle, g, _ptr(diag), _ptr(W), _stream(stream)),
               "trdq_layer_set_group")

    def forward(self, step, X, Y, bias=None, fused=False, Xq_ws=None, sx_ws=None, stream=None):
        """fused: True / False, or None to let the library choose (fused for few tokens)."""
        _check(lib().trdq_layer_forward(self.handle, step, _ptr(X), X.shape[0], _ptr(bias), _ptr(Y),
                                        -1 if fused is None else (1 if fused else 0), _ptr(Xq_ws), _ptr(sx_ws),
                                        _stream(stream)),
               "trdq_layer_forward")

    def weights(self, g):
        h = C.c_void_p()
        _check(lib().trdq_layer_weights(self.handle, g, C.byref(h)), "trdq_layer_weights")
        return Weights(h, owned=False)

    def close(self):
        if self.handle:
            lib().trdq_layer_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
