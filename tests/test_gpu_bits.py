"""GPU parity of the symmetric quantisers at other bit-widths (the W6A6 rows of Table 3):
trdq_rotate_quant_bits, trdq_prepare_weights(wbits=6) and the unchanged product on their codes."""
import numpy as np
import pytest
import torch

from paper_2503_06564_amd import trdq, workloads as wl
from gpu_util import (assert_codes_close, assert_scales_close, assert_y_close, assert_y_same_codes, narrow_code_masks, bf16_to_dev, bf16_to_host,
                      dev, f32_to_dev)

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def _rq_bits(Xbits, d, abits, warm=None):
    M, K = Xbits.shape
    Xq = torch.full((M, K), 99, dtype=torch.int8, device=dev())
    sx = torch.full((M,), -1.0, dtype=torch.float32, device=dev())
    trdq.rotate_quant_bits(bf16_to_dev(Xbits), f32_to_dev(d), Xq, sx, abits, warm=warm)
    torch.cuda.synchronize()
    return Xq, sx


@pytest.mark.parametrize("abits", [2, 4, 6, 7, 8])
@pytest.mark.parametrize("M,K", [(37, 256), (300, 1152), (64, 4608)])
def test_rotate_quant_bits_matches_oracle(oracle, M, K, abits):
    say(f"rotate_quant_bits M={M} K={K} abits={abits}")
    Xb, _, d, _ = wl.small_case(51, M, K, 16, n_outliers=max(1, K // 144), outlier=40.0)
    Xq, sx = _rq_bits(Xb, d, abits)
    Xq_o, sx_o = oracle.rotate_quant(Xb, d, 128, abits=abits)
    qmax = 2 ** (abits - 1) - 1
    q = Xq.cpu().numpy()
    assert np.abs(q).max() == qmax
    assert_codes_close(q, Xq_o, f"Xq ({abits} bits)")
    assert_scales_close(sx.cpu().numpy(), sx_o, f"s_x ({abits} bits)")


def test_rotate_quant_bits_8_is_rotate_quant(oracle):
    Xb, _, d, _ = wl.small_case(52, 515, 1152, 16, n_outliers=8)
    a, sa = _rq_bits(Xb, d, 8)
    Xq = torch.empty_like(a); sx = torch.empty_like(sa)
    trdq.rotate_quant(bf16_to_dev(Xb), f32_to_dev(d), Xq, sx)
    torch.cuda.synchronize()
    assert torch.equal(a, Xq) and torch.equal(sa, sx)


@pytest.mark.parametrize("M,K,N", [(17, 256, 144), (300, 1152, 272), (256, 1152, 288), (64, 384, 1152)])
@pytest.mark.parametrize("fused", [False, True])
def test_w6a6_linear_end_to_end(oracle, M, K, N, fused):
    say(f"W6A6 linear M={M} K={K} N={N} fused={fused}")
    Xb, W, d, bias = wl.small_case(53, M, K, N, n_outliers=max(1, K // 144), outlier=40.0)
    w = trdq.prepare_weights(f32_to_dev(W), f32_to_dev(d), wbits=6)
    assert w.info() == (K, N, 6)
    ref = oracle.linear(Xb, W, d, bias, wbits=6, abits=6, exact_blas=True)
    codes, scales = w.export()
    assert np.abs(codes).max() == 31
    assert_codes_close(codes, ref["Wq"], "Wq (6 bits)")
    assert_scales_close(scales, ref["sw"], "s_w (6 bits)")
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
    if fused:
        # the fused kernel quantises activations to 8 bits: W6A8
        trdq.linear_fused(bf16_to_dev(Xb), f32_to_dev(d), w, Y, bias=f32_to_dev(bias))
        torch.cuda.synchronize()
        ref68 = oracle.linear(Xb, W, d, bias, wbits=6, abits=8, exact_blas=True)
        assert_y_close(bf16_to_host(Y), ref68["Y"], "Y (W6A8 fused)")
    else:
        Xq, sx = _rq_bits(Xb, d, 6, warm=w)
        assert_codes_close(Xq.cpu().numpy(), ref["Xq"], "Xq (6 bits)")
        acc = torch.full((M, N), -7, dtype=torch.int32, device=dev())
        trdq.qgemm(w, Xq, sx, Y, bias=f32_to_dev(bias), acc_debug=acc)
        torch.cuda.synchronize()
        want = oracle.acc_exact_blas(Xq.cpu().numpy(), codes)
        assert np.array_equal(acc.cpu().numpy(), want)
        assert_y_close(bf16_to_host(Y), ref["Y"], "Y (W6A6)",
                       *narrow_code_masks(6, 6, Xq.cpu().numpy(), ref["Xq"], codes, ref["Wq"]))
        y_same = oracle.dequant(want, sx.cpu().numpy(), scales, bias)
        assert_y_same_codes(bf16_to_host(Y), y_same, "Y (W6A6, same codes)")
    w.close()


def test_rotate_quant_bits_rejects_bad_widths():
    X = torch.zeros((4, 256), dtype=torch.bfloat16, device=dev())
    Xq = torch.zeros((4, 256), dtype=torch.int8, device=dev())
    sx = torch.zeros((4,), device=dev())
    for bits in (1, 9, 0, -3):
        with pytest.raises(trdq.TrdqError) as e:
            trdq.rotate_quant_bits(X, None, Xq, sx, bits)
        assert e.value.status == trdq.ERR_RANGE
