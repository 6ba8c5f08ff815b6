"""GPU parity of the asymmetric activation quantiser of Eq. 1-3 (per-token zero point) and of the
product that carries it (trdq_rotate_quant_asym, trdq_qgemm_asym) against the oracle."""
import numpy as np
import pytest
import torch

from paper_2503_06564_amd import trdq, workloads as wl
from gpu_util import (assert_asym_codes_close, assert_codes_close, assert_scales_close, assert_y_close,
                      assert_y_same_codes, bf16_to_dev, bf16_to_host, dev, f32_to_dev, narrow_code_masks)

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def _gpu_rq_asym(Xbits, d, warm=None):
    M, K = Xbits.shape
    Xq = torch.full((M, K), 99, dtype=torch.int8, device=dev())
    sx = torch.full((M,), -1.0, dtype=torch.float32, device=dev())
    zc = torch.full((M,), -999, dtype=torch.int32, device=dev())
    trdq.rotate_quant_asym(bf16_to_dev(Xbits), f32_to_dev(d), Xq, sx, zc, warm=warm)
    torch.cuda.synchronize()
    return Xq, sx, zc


def _compare_codes(oracle, Xb, d, Xq, sx, zc):
    """codes (relative to their zero point), zero points and scales against the oracle"""
    Xq_o, sx_o, zx_o = oracle.quant_tokens_asym(oracle.rotate(Xb, d, 128))
    q = Xq.cpu().numpy().astype(np.int16) + 128
    z = 128 - zc.cpu().numpy()
    assert_asym_codes_close(q, z, Xq_o, zx_o, "Xq (asymmetric)")
    assert_scales_close(sx.cpu().numpy(), sx_o, "s_x (asymmetric)")


@pytest.mark.parametrize("M,K", [(1, 128), (37, 256), (300, 1152), (64, 4608), (2048, 1152), (0, 256)])
def test_rotate_quant_asym_matches_oracle(oracle, M, K):
    say(f"rotate_quant_asym M={M} K={K}")
    Xb, W, d, bias = wl.small_case(41, max(M, 1), K, 16, n_outliers=max(1, K // 144), outlier=40.0)
    Xb = Xb[:M]
    Xq, sx, zc = _gpu_rq_asym(Xb, d)
    if M:
        _compare_codes(oracle, Xb, d, Xq, sx, zc)


def test_rotate_quant_asym_one_sided_and_zero_rows(oracle):
    K = 256
    x = np.zeros((4, K), dtype=np.float32)
    x[0, 0] = 3.0                      # after the rotation: +-3/sqrt(128) in block 0, zeros elsewhere
    x[1, :] = 0.0                      # all zeros
    x[2, :128] = 1.0                   # constant block: one positive coefficient, the rest zero
    x[3, :128] = -2.0                  # one negative coefficient: hi = 0, z = 255
    Xb = wl.f32_to_bf16_bits(x)
    Xq, sx, zc = _gpu_rq_asym(Xb, None)
    Xq_o, sx_o, zx_o = oracle.quant_tokens_asym(oracle.rotate(Xb, None, 128))
    assert np.array_equal(128 - zc.cpu().numpy(), zx_o)
    assert np.array_equal(Xq.cpu().numpy().astype(np.int16) + 128, Xq_o)
    assert_scales_close(sx.cpu().numpy(), sx_o, "s_x")
    assert sx[1].item() == 0.0 and zx_o[2] == 0 and zx_o[3] == 255


# the last five shapes reach the 128 x 144 kernels: one workgroup per tile (K < 2304), two wave groups
# splitting K (even and odd numbers of k-tiles), two workgroups per compute unit (more than 256 tiles)
@pytest.mark.parametrize("M,K,N", [(1, 128, 16), (17, 256, 144), (300, 4608, 272), (513, 384, 400), (1024, 1152, 1152),
                                   (256, 1152, 288), (256, 2304, 144), (384, 4608, 144), (256, 2432, 144),
                                   (4224, 512, 1152), (1100, 1152, 1152), (1407, 2304, 144)])
def test_linear_asym_end_to_end(oracle, M, K, N):
    say(f"linear asymmetric M={M} K={K} N={N}")
    Xb, W, d, bias = wl.small_case(42, M, K, N, n_outliers=max(1, K // 144), outlier=40.0)
    w = trdq.prepare_weights(f32_to_dev(W), f32_to_dev(d), wbits=8)
    Xq, sx, zc = _gpu_rq_asym(Xb, d, warm=w)
    _compare_codes(oracle, Xb, d, Xq, sx, zc)
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
    acc = torch.full((M, N), -7, dtype=torch.int32, device=dev())
    trdq.qgemm_asym(w, Xq, sx, zc, Y, bias=f32_to_dev(bias), acc_debug=acc)
    torch.cuda.synchronize()
    codes, scales = w.export()
    q = (Xq.cpu().numpy().astype(np.int16) + 128).astype(np.uint8)
    z = (128 - zc.cpu().numpy()).astype(np.int32)
    want_acc = oracle.acc_asym_exact_blas(q, z, codes)
    assert np.array_equal(acc.cpu().numpy(), want_acc), "integer sums differ on the GPU's own codes"
    y_same = oracle.dequant(want_acc, sx.cpu().numpy(), scales, bias)
    assert_y_same_codes(bf16_to_host(Y), y_same, "Y (same codes)")
    ref = oracle.linear_asym(Xb, W, d, bias, exact_blas=True)
    assert_codes_close(codes, ref["Wq"], "Wq")
    assert_y_close(bf16_to_host(Y), ref["Y"], "Y (oracle end to end)")
    Y2 = torch.zeros_like(Y)
    trdq.qgemm_asym(w, Xq, sx, zc, Y2, bias=f32_to_dev(bias))
    torch.cuda.synchronize()
    assert torch.equal(Y2, Y)
    w.close()


@pytest.mark.parametrize("M,K,N", [(1, 128, 16), (17, 256, 144), (300, 4608, 272), (513, 384, 400), (1024, 1152, 1152)])
def test_linear_asym_int4_weights(oracle, M, K, N):
    say(f"linear asymmetric W4 M={M} K={K} N={N}")
    Xb, W, d, bias = wl.small_case(43, M, K, N, n_outliers=max(1, K // 144), outlier=40.0)
    w = trdq.prepare_weights(f32_to_dev(W), f32_to_dev(d), wbits=4)
    Xq, sx, zc = _gpu_rq_asym(Xb, d, warm=w)
    _compare_codes(oracle, Xb, d, Xq, sx, zc)
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
    trdq.qgemm_asym(w, Xq, sx, zc, Y, bias=f32_to_dev(bias))
    torch.cuda.synchronize()
    codes, scales = w.export()
    q = (Xq.cpu().numpy().astype(np.int16) + 128).astype(np.uint8)
    z = (128 - zc.cpu().numpy()).astype(np.int32)
    # the oracle's epilogue on the GPU's own codes and zero points
    acc = oracle.igemm_asym_groups(q, z, codes, 128, exact_blas=True)
    y_same = oracle.dequant(acc, sx.cpu().numpy(), scales, bias)
    # fp32 group sums and a float zero-point term that cancels part of them: one bf16 step plus 1e-4 of the row's magnitude
    assert_y_same_codes(bf16_to_host(Y), y_same, "Y (asymmetric, int4 weights, same codes)", rel=1e-4)
    ref = oracle.linear_asym(Xb, W, d, bias, exact_blas=True, wbits=4)
    assert_codes_close(codes, ref["Wq"], "Wq (int4)")
    assert_y_close(bf16_to_host(Y), ref["Y"], "Y (asymmetric, int4 weights)",
                   *narrow_code_masks(8, 4, None, None, codes, ref["Wq"]))
    w.close()


# both fused kernels: few tokens (one 16-token panel per workgroup, K <= 1536) and the general one
# (panels of 64, 32 and 16 tokens as K grows); ragged token and channel counts, with and without a diagonal
@pytest.mark.parametrize("M,K,N,wbits", [(1, 128, 16, 8), (17, 256, 144, 8), (256, 1152, 1152, 8), (100, 1152, 272, 6),
                                         (1100, 1152, 1152, 8), (513, 384, 400, 8), (300, 2304, 272, 8),
                                         (200, 4608, 144, 8), (1024, 1152, 3456, 6)])
def test_linear_fused_asym_matches_oracle(oracle, M, K, N, wbits):
    say(f"linear fused asymmetric M={M} K={K} N={N} wbits={wbits}")
    Xb, W, d, bias = wl.small_case(45, M, K, N, n_outliers=max(1, K // 144), outlier=40.0)
    w = trdq.prepare_weights(f32_to_dev(W), f32_to_dev(d), wbits=wbits)
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
    trdq.linear_fused_asym(bf16_to_dev(Xb), f32_to_dev(d), w, Y, bias=f32_to_dev(bias))
    torch.cuda.synchronize()
    codes, _ = w.export()
    ref = oracle.linear_asym(Xb, W, d, bias, exact_blas=True, wbits=wbits)
    assert_y_close(bf16_to_host(Y), ref["Y"], "Y (fused, asymmetric, oracle end to end)",
                   *narrow_code_masks(8, wbits, None, None, codes, ref["Wq"]))
    # the unfused pair on the same inputs: same arithmetic up to the rounding order of the rotation
    Xq, sx, zc = _gpu_rq_asym(Xb, d)
    Yp = torch.zeros_like(Y)
    trdq.qgemm_asym(w, Xq, sx, zc, Yp, bias=f32_to_dev(bias))
    torch.cuda.synchronize()
    assert_y_close(bf16_to_host(Y), bf16_to_host(Yp), "Y (fused against the pair)")
    w.close()


def test_linear_fused_asym_without_diagonal_and_one_sided_rows(oracle):
    K, N = 256, 144
    x = np.zeros((5, K), dtype=np.float32)
    x[0, 0] = 3.0
    x[2, :128] = 1.0
    x[3, :128] = -2.0
    x[4] = np.linspace(-1.0, 2.0, K)
    Xb = wl.f32_to_bf16_bits(x)
    _, W, _, bias = wl.small_case(46, 5, K, N)
    w = trdq.prepare_weights(f32_to_dev(W), None, wbits=8)
    Y = torch.full((5, N), 7.0, dtype=torch.bfloat16, device=dev())
    trdq.linear_fused_asym(bf16_to_dev(Xb), None, w, Y, bias=f32_to_dev(bias))
    torch.cuda.synchronize()
    ref = oracle.linear_asym(Xb, W, None, bias, exact_blas=True)
    assert_y_close(bf16_to_host(Y), ref["Y"], "Y (fused, asymmetric, special rows)")
    # the all-zero token yields the bias alone
    assert np.array_equal(bf16_to_host(Y)[1], wl.f32_to_bf16_bits(bias.astype(np.float32)))
    w.close()


def test_linear_fused_asym_refusals():
    _, W, d, _ = wl.small_case(47, 4, 256, 32)
    X = torch.zeros((4, 256), dtype=torch.bfloat16, device=dev())
    Y = torch.zeros((4, 32), dtype=torch.bfloat16, device=dev())
    w4 = trdq.prepare_weights(f32_to_dev(W), f32_to_dev(d), wbits=4)
    with pytest.raises(trdq.TrdqError) as e:
        trdq.linear_fused_asym(X, f32_to_dev(d), w4, Y)
    assert e.value.status == trdq.ERR_UNSUPPORTED
    w4.close()
    wa = trdq.prepare_weights_asym(f32_to_dev(W), f32_to_dev(d))
    with pytest.raises(trdq.TrdqError) as e:
        trdq.linear_fused_asym(X, f32_to_dev(d), wa, Y)
    assert e.value.status == trdq.ERR_MISMATCH
    wa.close()
