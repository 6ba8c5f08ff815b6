"""GPU parity of the full transform of Eq. 9 (rotation, zigzag permutation, rotation).

trdq_zigzag_permutation, trdq_prepare_weights_rpr and trdq_rotate_quant_rpr against the oracle's
dense float64 G_t = X D R P R and H_t = R^T P^T R^T D^-1 W, to the same bars as the one-rotation
path: codes within one LSB on <= 0.01 % of elements, scales to 1e-5, int32 sums bit-exact on the
GPU's own codes, bf16 outputs within 1e-2 x row absmax.
"""
import numpy as np
import pytest
import torch

from paper_2503_06564_amd import trdq, workloads as wl
from gpu_util import (assert_codes_close, assert_scales_close, assert_y_close, assert_y_same_codes, narrow_code_masks, bf16_to_dev, bf16_to_host,
                      dev, f32_to_dev, gpu_qgemm)

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def _perm_for(oracle, Xb, d, B=128):
    """Zigzag permutation from the per-channel absmax of the once-rotated activations (host)."""
    V1 = oracle.rotate(Xb, d, B)
    return np.abs(V1).max(axis=0)


def _gpu_rotate_quant_rpr(Xbits, d, perm, ldx=None):
    M, K = Xbits.shape
    if ldx is None:
        X = bf16_to_dev(Xbits)
    else:
        buf = torch.zeros((max(M, 1), ldx), dtype=torch.bfloat16, device=dev())
        X = buf[:M, :K]
        X.copy_(bf16_to_dev(Xbits))
    Xq = torch.full((M, K), 99, dtype=torch.int8, device=dev())
    sx = torch.full((M,), -1.0, dtype=torch.float32, device=dev())
    perm_d = torch.from_numpy(np.ascontiguousarray(perm, dtype=np.int32)).to(dev())
    trdq.rotate_quant_rpr(X, f32_to_dev(d), perm_d, Xq, sx)
    torch.cuda.synchronize()
    return Xq, sx


# (M, K): one block, the DiT widths (16 tokens per workgroup up to K = 2304, 8 above), ragged M
RPR_SHAPES = [(16, 128), (37, 256), (64, 1152), (21, 2304), (40, 2432), (19, 4608), (1, 1152), (0, 1152)]


@pytest.mark.parametrize("M,K", RPR_SHAPES)
def test_rotate_quant_rpr_matches_oracle(oracle, M, K):
    say(f"rotate_quant_rpr M={M} K={K}")
    Xb, W, d, bias = wl.small_case(21, max(M, 1), K, 16, n_outliers=max(1, K // 144), outlier=40.0)
    Xb = Xb[:M]
    ref_rows = Xb if M > 0 else wl.small_case(21, 4, K, 16)[0]
    perm = trdq.zigzag_permutation(_perm_for(oracle, ref_rows, d).astype(np.float32))
    Xq, sx = _gpu_rotate_quant_rpr(Xb, d, perm)
    if M == 0:
        return
    Xq_o, sx_o = oracle.rotate_quant_rpr(Xb, d, perm, 128)
    assert_codes_close(Xq.cpu().numpy(), Xq_o, "Xq (R P R)")
    assert_scales_close(sx.cpu().numpy(), sx_o, "s_x (R P R)")


def test_rotate_quant_rpr_strided_rows_and_no_diag(oracle):
    M, K = 33, 1152
    Xb, *_ = wl.small_case(22, M, K, 16, n_outliers=8, outlier=50.0)
    rng = np.random.default_rng(3)
    perm = rng.permutation(K).astype(np.int32)                  # any permutation, not only a zigzag
    Xq, sx = _gpu_rotate_quant_rpr(Xb, None, perm, ldx=K + 64)
    Xq_o, sx_o = oracle.rotate_quant_rpr(Xb, None, perm, 128)
    assert_codes_close(Xq.cpu().numpy(), Xq_o, "Xq (strided, no diagonal)")
    assert_scales_close(sx.cpu().numpy(), sx_o, "s_x (strided, no diagonal)")


def test_rpr_identity_permutation_is_plain_scaling(oracle):
    # R R = I: with P = I the transform is X diag(d); the codes are those of quantising that
    M, K = 16, 1152
    Xb, W, d, *_ = wl.small_case(23, M, K, 16, n_outliers=8, outlier=50.0)
    Xq, sx = _gpu_rotate_quant_rpr(Xb, d, np.arange(K, dtype=np.int32))
    U = oracle.bf16_to_f64(Xb) * d.astype(np.float64)
    Xq_o, sx_o = oracle.quant_tokens(U)
    assert_codes_close(Xq.cpu().numpy(), Xq_o, "Xq (identity permutation)")
    assert_scales_close(sx.cpu().numpy(), sx_o, "s_x (identity permutation)")


@pytest.mark.parametrize("wbits", [8, 4])
@pytest.mark.parametrize("M,K,N", [(48, 256, 32), (130, 1152, 288), (64, 4608, 144)])
def test_linear_rpr_end_to_end(oracle, M, K, N, wbits):
    say(f"linear R P R M={M} K={K} N={N} W{wbits}")
    Xb, W, d, bias = wl.small_case(24, M, K, N, n_outliers=max(1, K // 144), outlier=40.0)
    perm = trdq.zigzag_permutation(_perm_for(oracle, Xb, d).astype(np.float32))
    perm_d = torch.from_numpy(perm).to(dev())
    w = trdq.prepare_weights_rpr(f32_to_dev(W), f32_to_dev(d), perm_d, wbits=wbits)
    codes, scales = w.export()
    Wq_o, sw_o = oracle.prepare_weights_rpr(W, d, perm, 128, wbits)
    assert_codes_close(codes, Wq_o, "Wq (R P R)")
    assert_scales_close(scales, sw_o, "s_w (R P R)")

    Xq, sx = _gpu_rotate_quant_rpr(Xb, d, perm)
    Xq_o, sx_o = oracle.rotate_quant_rpr(Xb, d, perm, 128)
    assert_codes_close(Xq.cpu().numpy(), Xq_o, "Xq (R P R)")

    Y, acc = gpu_qgemm(w, Xq, sx, bias, N)
    group = None if wbits == 8 else 128
    acc_o = oracle.acc_exact_blas(Xq.cpu().numpy(), codes, group)
    assert np.array_equal(acc.cpu().numpy(), acc_o), "int32 sums differ on the GPU's own codes"
    ref = oracle.linear_rpr(Xb, W, d, perm, bias, 128, wbits, exact_blas=True)
    assert_y_close(bf16_to_host(Y), ref["Y"], "Y (R P R)", *narrow_code_masks(8, wbits, None, None, codes, ref["Wq"]))
    y_same = oracle.dequant(acc_o, sx.cpu().numpy(), scales, bias)
    assert_y_same_codes(bf16_to_host(Y), y_same, "Y (R P R, same codes)")
    # the product is unchanged by the transform (Eq. 9): close to the unquantised X W + bias
    exact = oracle.bf16_to_f64(Xb) @ W.astype(np.float64) + bias.astype(np.float64)
    got = oracle.bf16_to_f64(bf16_to_host(Y))
    rel = np.linalg.norm(got - exact) / np.linalg.norm(exact)
    assert rel < (0.03 if wbits == 8 else 0.2), rel


# ---- calibration side: channel statistics and Eq. 5 --------------------------------------------

@pytest.mark.parametrize("M,K", [(1, 128), (37, 256), (300, 1152), (4096, 1152), (1000, 4608)])
@pytest.mark.parametrize("rotate", [False, True])
def test_channel_absmax_matches_oracle(oracle, M, K, rotate):
    say(f"channel_absmax M={M} K={K} rotate={rotate}")
    Xb, W, d, bias = wl.small_case(31, M, K, 16, n_outliers=max(1, K // 144), outlier=40.0)
    mag = torch.full((K,), -1.0, dtype=torch.float32, device=dev())
    trdq.channel_absmax(bf16_to_dev(Xb), f32_to_dev(d), mag, rotate=rotate)
    torch.cuda.synchronize()
    want = oracle.channel_absmax(Xb, d, rotate_first=rotate)
    assert np.allclose(mag.cpu().numpy(), want, rtol=1e-5, atol=0)
    # no diagonal, strided rows
    buf = torch.zeros((M, K + 64), dtype=torch.bfloat16, device=dev())
    Xs = buf[:, :K]
    Xs.copy_(bf16_to_dev(Xb))
    trdq.channel_absmax(Xs, None, mag, rotate=rotate)
    torch.cuda.synchronize()
    assert np.allclose(mag.cpu().numpy(), oracle.channel_absmax(Xb, None, rotate_first=rotate), rtol=1e-5, atol=0)


def test_channel_absmax_no_tokens_gives_zeros():
    mag = torch.full((256,), -1.0, dtype=torch.float32, device=dev())
    X = torch.empty((0, 256), dtype=torch.bfloat16, device=dev())
    trdq.channel_absmax(X, None, mag, rotate=True)
    torch.cuda.synchronize()
    assert bool((mag == 0).all())


@pytest.mark.parametrize("alpha", [0.0, 0.5, 0.85, 1.0])
def test_smoothing_diagonal_matches_oracle(oracle, alpha):
    M, K, N = 256, 1152, 272
    Xb, W, d, bias = wl.small_case(32, M, K, N, n_outliers=8, outlier=50.0)
    W[5] = 0.0                                                    # a dead weight row: d = 1 there
    xmax = torch.empty((K,), dtype=torch.float32, device=dev())
    wmax = torch.empty((K,), dtype=torch.float32, device=dev())
    diag = torch.empty((K,), dtype=torch.float32, device=dev())
    trdq.channel_absmax(bf16_to_dev(Xb), None, xmax)
    trdq.weight_row_absmax(f32_to_dev(W), wmax)
    trdq.smooth_diag(xmax, wmax, alpha, diag)
    torch.cuda.synchronize()
    xo, wo = oracle.channel_absmax(Xb), oracle.weight_row_absmax(W)
    assert np.array_equal(xmax.cpu().numpy().astype(np.float64), xo)          # maxima of bf16 values: exact
    assert np.array_equal(wmax.cpu().numpy().astype(np.float64), wo)
    want = oracle.smooth_diag(xo, wo, alpha)
    assert np.allclose(diag.cpu().numpy(), want, rtol=1e-5, atol=0)
    assert diag[5].item() == 1.0


def test_calibrate_then_run_the_full_path(oracle):
    """Eq. 5 diagonal and zigzag permutation computed on the GPU from the data, then the Eq. 9 path."""
    M, K, N = 192, 1152, 288
    Xb, W, _, bias = wl.small_case(33, M, K, N, n_outliers=8, outlier=50.0)
    X, Wd = bf16_to_dev(Xb), f32_to_dev(W)
    xmax = torch.empty((K,), dtype=torch.float32, device=dev())
    wmax = torch.empty_like(xmax)
    diag = torch.empty_like(xmax)
    mag = torch.empty_like(xmax)
    trdq.channel_absmax(X, None, xmax)
    trdq.weight_row_absmax(Wd, wmax)
    trdq.smooth_diag(xmax, wmax, 0.5, diag)
    trdq.channel_absmax(X, diag, mag, rotate=True)
    torch.cuda.synchronize()
    d = diag.cpu().numpy()
    perm = trdq.zigzag_permutation(mag.cpu().numpy())
    perm_d = torch.from_numpy(perm).to(dev())
    w = trdq.prepare_weights_rpr(Wd, diag, perm_d, wbits=8)
    Xq, sx = _gpu_rotate_quant_rpr(Xb, d, perm)
    Y, _ = gpu_qgemm(w, Xq, sx, bias, N, debug=False)
    ref = oracle.linear_rpr(Xb, W, d, perm, bias, 128, 8, exact_blas=True)
    codes, _ = w.export()
    assert_codes_close(Xq.cpu().numpy(), ref["Xq"], "Xq (calibrated R P R)")
    assert_codes_close(codes, ref["Wq"], "Wq (calibrated R P R)")
    assert_y_close(bf16_to_host(Y), ref["Y"], "Y (calibrated R P R)")
    exact = oracle.bf16_to_f64(Xb) @ W.astype(np.float64) + bias.astype(np.float64)
    got = oracle.bf16_to_f64(bf16_to_host(Y))
    assert np.linalg.norm(got - exact) / np.linalg.norm(exact) < 0.03


def test_fused_refuses_weights_folded_with_another_transform(oracle):
    """The fused kernel applies the one-rotation transform: weights folded with R P R (or dense blocks)
    are refused instead of multiplied with the wrong activations."""
    M, K, N = 32, 256, 144
    Xb, W, d, bias = wl.small_case(29, M, K, N)
    perm_d = torch.from_numpy(oracle.zigzag(np.arange(K, dtype=np.float64), 128).astype(np.int32)).to(dev())
    w = trdq.prepare_weights_rpr(f32_to_dev(W), f32_to_dev(d), perm_d, wbits=8)
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
    with pytest.raises(trdq.TrdqError) as e:
        trdq.linear_fused(bf16_to_dev(Xb), f32_to_dev(d), w, Y)
    assert e.value.status == trdq.ERR_MISMATCH
    w.close()


@pytest.mark.parametrize("M,K,N", [(17, 256, 144), (300, 1152, 272), (130, 4608, 144), (1024, 1152, 1152)])
def test_rpr_with_asymmetric_activation_codes(oracle, M, K, N):
    """Eq. 9's transform followed by the asymmetric quantiser of Eq. 1-3 (trdq_rotate_quant_rpr_asym), multiplied
    by trdq_qgemm_asym against weights from trdq_prepare_weights_rpr."""
    say(f"R P R, asymmetric codes M={M} K={K} N={N}")
    from gpu_util import assert_asym_codes_close
    Xb, W, d, bias = wl.small_case(26, M, K, N, n_outliers=max(1, K // 144), outlier=40.0)
    perm = trdq.zigzag_permutation(_perm_for(oracle, Xb, d).astype(np.float32))
    perm_d = torch.from_numpy(perm).to(dev())
    w = trdq.prepare_weights_rpr(f32_to_dev(W), f32_to_dev(d), perm_d, wbits=8)
    Xq = torch.full((M, K), 99, dtype=torch.int8, device=dev())
    sx = torch.full((M,), -1.0, dtype=torch.float32, device=dev())
    zc = torch.full((M,), -999, dtype=torch.int32, device=dev())
    trdq.rotate_quant_rpr_asym(bf16_to_dev(Xb), f32_to_dev(d), perm_d, Xq, sx, zc, warm=w)
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
    acc = torch.full((M, N), -7, dtype=torch.int32, device=dev())
    trdq.qgemm_asym(w, Xq, sx, zc, Y, bias=f32_to_dev(bias), acc_debug=acc)
    torch.cuda.synchronize()
    ref = oracle.linear_rpr_asym(Xb, W, d, perm, bias, exact_blas=True)
    q = Xq.cpu().numpy().astype(np.int16) + 128
    z = (128 - zc.cpu().numpy()).astype(np.int32)
    assert_asym_codes_close(q, z, ref["Xq"], ref["zx"], "Xq (R P R, asymmetric)")
    assert_scales_close(sx.cpu().numpy(), ref["sx"], "s_x (R P R, asymmetric)")
    codes, scales = w.export()
    assert_codes_close(codes, ref["Wq"], "Wq (R P R)")
    want = oracle.acc_asym_exact_blas(q.astype(np.uint8), z, codes)
    assert np.array_equal(acc.cpu().numpy(), want), "integer sums differ on the GPU's own codes"
    assert_y_same_codes(bf16_to_host(Y), oracle.dequant(want, sx.cpu().numpy(), scales, bias), "Y (same codes)")
    assert_y_close(bf16_to_host(Y), ref["Y"], "Y (R P R, asymmetric)")
    # the symmetric pass is untouched by the new option: bits of the plain call
    Xq2, sx2 = _gpu_rotate_quant_rpr(Xb, d, perm)
    Xq_o, sx_o = oracle.rotate_quant_rpr(Xb, d, perm, 128)
    assert_codes_close(Xq2.cpu().numpy(), Xq_o, "Xq (R P R, symmetric)")
    w.close()
