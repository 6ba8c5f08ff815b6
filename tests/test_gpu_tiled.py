"""GPU parity of the pair on block-tiled activation codes (trdq_rotate_quant_tiled, trdq_qgemm_tiled)
against the oracle and against the row-major pair: the tiled codes are the row-major codes moved,
the integer sums are exact, the epilogue is the same arithmetic."""
import numpy as np
import pytest
import torch

from paper_2503_06564_amd import trdq, workloads as wl
from gpu_util import (narrow_code_masks, assert_codes_close, assert_scales_close, assert_y_close, assert_y_same_codes, bf16_to_dev,
                      bf16_to_host, dev, f32_to_dev)

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def tile_host(a):
    """[M, K] int8 (M % 16 == 0) -> the block-tiled byte order, on the host, from the stated formula."""
    M, K = a.shape
    # [row group][row][k block][piece][16 bytes] -> [row group][k block][piece][row][16 bytes]
    return np.ascontiguousarray(a.reshape(M // 16, 16, K // 64, 4, 16).transpose(0, 2, 3, 1, 4)).reshape(-1)


@pytest.mark.parametrize("M,K", [(16, 128), (37, 256), (128, 1152), (1000, 1152), (130, 4608), (4096, 1152)])
def test_rotate_quant_tiled_is_rotate_quant_moved(oracle, M, K):
    say(f"rotate_quant_tiled M={M} K={K}")
    Xb, _, d, _ = wl.small_case(71, M, K, 16, n_outliers=max(1, K // 144))
    X, dd = bf16_to_dev(Xb), f32_to_dev(d)
    Xq = torch.empty((M, K), dtype=torch.int8, device=dev())
    sx = torch.empty((M,), dtype=torch.float32, device=dev())
    trdq.rotate_quant(X, dd, Xq, sx)
    nbytes = trdq.xq_tiled_nbytes(M, K)
    assert nbytes == (M + 15) // 16 * 16 * K
    Xt = torch.full((nbytes,), 99, dtype=torch.int8, device=dev())
    sxt = torch.empty((M,), dtype=torch.float32, device=dev())
    trdq.rotate_quant_tiled(X, dd, Xt, sxt)
    back = torch.full((M, K), -99, dtype=torch.int8, device=dev())
    trdq.xq_untile(Xt, M, K, back)
    torch.cuda.synchronize()
    assert torch.equal(back, Xq) and torch.equal(sxt, sx)
    # the byte order itself, from the formula of the interface, on whole groups of 16 tokens
    Mw = M // 16 * 16
    assert np.array_equal(Xt.cpu().numpy()[:Mw * K], tile_host(Xq.cpu().numpy()[:Mw]))
    want_q, want_s = oracle.rotate_quant(Xb, d)
    assert_codes_close(back.cpu().numpy(), want_q, "Xq (tiled)")
    assert_scales_close(sxt.cpu().numpy(), want_s, "s_x (tiled)")


# tall tiles only, short tiles only, both in one launch (more short tiles than two per compute unit),
# one and several k-step pairs, the real layer widths
# the last five reach the kernel that splits K over four wave pairs (at most one 128 x 144 tile per compute
# unit, K a multiple of 512): two, four and six k-steps per pair, one tile and a full round of tiles
TILED_SHAPES = [(128, 128, 144), (256, 256, 144), (384, 384, 288), (1024, 1152, 1152), (4096, 128, 3456),
                (4096, 1152, 3456), (2048, 4608, 1152), (8192, 256, 1152), (3840, 640, 2304),
                (128, 1024, 144), (256, 1024, 288), (384, 1536, 144), (1152, 2048, 432), (256, 1280, 144), (256, 1152, 288), (4096, 4608, 1152)]


@pytest.mark.parametrize("M,K,N", TILED_SHAPES)
@pytest.mark.parametrize("with_bias", [True, False])
def test_qgemm_tiled_matches_oracle(oracle, M, K, N, with_bias):
    say(f"qgemm_tiled M={M} K={K} N={N} bias={with_bias}")
    Xb, W, d, bias = wl.small_case(72, M, K, N, n_outliers=max(1, K // 144))
    bias = bias if with_bias else None
    w = trdq.prepare_weights(f32_to_dev(W), f32_to_dev(d), wbits=8)
    assert trdq.qgemm_tiled_supported(w, M)
    X, dd = bf16_to_dev(Xb), f32_to_dev(d)
    Xt = torch.empty((trdq.xq_tiled_nbytes(M, K),), dtype=torch.int8, device=dev())
    sx = torch.empty((M,), dtype=torch.float32, device=dev())
    trdq.rotate_quant_tiled(X, dd, Xt, sx, warm=w)
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
    acc = torch.full((M, N), -7, dtype=torch.int32, device=dev())
    trdq.qgemm_tiled(w, Xt, sx, Y, bias=f32_to_dev(bias), acc_debug=acc)
    Xq = torch.empty((M, K), dtype=torch.int8, device=dev())
    trdq.xq_untile(Xt, M, K, Xq)
    torch.cuda.synchronize()
    Xq_h, (Wq_h, sw_h) = Xq.cpu().numpy(), w.export()
    # integer sums bit-exact on the GPU's own codes
    want_acc = oracle.acc_exact_blas(Xq_h, Wq_h)
    assert np.array_equal(acc.cpu().numpy(), want_acc), "int32 accumulators differ"
    y_same = oracle.dequant(want_acc, sx.cpu().numpy(), sw_h, bias)
    assert_y_same_codes(bf16_to_host(Y), y_same, "Y (same codes)")
    ref = oracle.linear(Xb, W, d, bias, wbits=8, exact_blas=True)
    assert_codes_close(Xq_h, ref["Xq"], "Xq")
    assert_codes_close(Wq_h, ref["Wq"], "Wq")
    assert_y_close(bf16_to_host(Y), ref["Y"], "Y (oracle end to end)")
    # without the debug output, and against the row-major pair: the same bits
    Y2 = torch.zeros_like(Y)
    trdq.qgemm_tiled(w, Xt, sx, Y2, bias=f32_to_dev(bias))
    Y3 = torch.zeros_like(Y)
    trdq.qgemm(w, Xq, sx, Y3, bias=f32_to_dev(bias))
    torch.cuda.synchronize()
    assert torch.equal(Y2, Y)
    assert torch.equal(Y3, Y), "tiled and row-major products differ"
    w.close()


# int4 weights: 128 x 128 tiles, three scale groups (the least the kernel takes), ragged counts of tiles per
# compute unit, the real layer widths
TILED4_SHAPES = [(128, 384, 128), (256, 512, 256), (384, 1152, 1152), (1024, 4608, 1152), (4096, 1152, 3456),
                 (2048, 640, 4608)]


@pytest.mark.parametrize("M,K,N", TILED4_SHAPES)
@pytest.mark.parametrize("with_bias", [True, False])
def test_qgemm_tiled_int4_matches_oracle(oracle, M, K, N, with_bias):
    say(f"qgemm_tiled int4 M={M} K={K} N={N} bias={with_bias}")
    Xb, W, d, bias = wl.small_case(75, M, K, N, n_outliers=max(1, K // 144))
    bias = bias if with_bias else None
    w = trdq.prepare_weights(f32_to_dev(W), f32_to_dev(d), wbits=4)
    assert trdq.qgemm_tiled_supported(w, M)
    X, dd = bf16_to_dev(Xb), f32_to_dev(d)
    Xt = torch.empty((trdq.xq_tiled_nbytes(M, K),), dtype=torch.int8, device=dev())
    sx = torch.empty((M,), dtype=torch.float32, device=dev())
    trdq.rotate_quant_tiled(X, dd, Xt, sx, warm=w)
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
    acc = torch.full((K // 128, M, N), -7, dtype=torch.int32, device=dev())
    trdq.qgemm_tiled(w, Xt, sx, Y, bias=f32_to_dev(bias), acc_debug=acc)
    Xq = torch.empty((M, K), dtype=torch.int8, device=dev())
    trdq.xq_untile(Xt, M, K, Xq)
    torch.cuda.synchronize()
    Xq_h, (Wq_h, sw_h) = Xq.cpu().numpy(), w.export()
    # the per-group integer sums, bit-exact on the GPU's own codes
    want_acc = oracle.acc_exact_blas(Xq_h, Wq_h, 128)
    assert np.array_equal(acc.cpu().numpy(), want_acc), "int32 group sums differ"
    y_same = oracle.dequant(want_acc, sx.cpu().numpy(), sw_h, bias)
    assert_y_same_codes(bf16_to_host(Y), y_same, "Y (int4, same codes)")
    ref = oracle.linear(Xb, W, d, bias, wbits=4, exact_blas=True)
    assert_codes_close(Xq_h, ref["Xq"], "Xq")
    assert_codes_close(Wq_h, ref["Wq"], "Wq (int4)")
    assert_y_close(bf16_to_host(Y), ref["Y"], "Y (int4, oracle end to end)",
                   *narrow_code_masks(8, 4, None, None, Wq_h, ref["Wq"]))
    # without the debug output, and against the row-major pair: the same bits (same order of the float folds)
    Y2 = torch.zeros_like(Y)
    trdq.qgemm_tiled(w, Xt, sx, Y2, bias=f32_to_dev(bias))
    Y3 = torch.zeros_like(Y)
    trdq.qgemm(w, Xq, sx, Y3, bias=f32_to_dev(bias))
    torch.cuda.synchronize()
    assert torch.equal(Y2, Y)
    assert torch.equal(Y3, Y), "tiled and row-major int4 products differ"
    w.close()


def test_qgemm_tiled_int4_refuses_what_it_does_not_take():
    _, W, d, _ = wl.small_case(76, 4, 256, 128)
    w = trdq.prepare_weights(f32_to_dev(W), f32_to_dev(d), wbits=4)              # two scale groups: too short
    assert not trdq.qgemm_tiled_supported(w, 128)
    Xt = torch.zeros((128 * 256,), dtype=torch.int8, device=dev())
    sx = torch.ones((128,), dtype=torch.float32, device=dev())
    Y = torch.zeros((128, 128), dtype=torch.bfloat16, device=dev())
    with pytest.raises(trdq.TrdqError) as e:
        trdq.qgemm_tiled(w, Xt, sx, Y)
    assert e.value.status == trdq.ERR_UNSUPPORTED
    w.close()


def test_qgemm_tiled_refuses_what_it_does_not_take(oracle):
    _, W, d, _ = wl.small_case(73, 4, 256, 160)
    w160 = trdq.prepare_weights(f32_to_dev(W), f32_to_dev(d), wbits=8)          # 160 is not a multiple of 144
    _, W, d, _ = wl.small_case(73, 4, 256, 144)
    w4 = trdq.prepare_weights(f32_to_dev(W), f32_to_dev(d), wbits=4)            # int4 weights
    w8 = trdq.prepare_weights(f32_to_dev(W), f32_to_dev(d), wbits=8)
    assert not trdq.qgemm_tiled_supported(w160, 128) and not trdq.qgemm_tiled_supported(w4, 128)
    assert trdq.qgemm_tiled_supported(w8, 128) and not trdq.qgemm_tiled_supported(w8, 100)
    Xt = torch.zeros((128 * 256,), dtype=torch.int8, device=dev())
    sx = torch.ones((128,), dtype=torch.float32, device=dev())
    for w, M, N in ((w160, 128, 160), (w4, 128, 144), (w8, 112, 144)):
        Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
        with pytest.raises(trdq.TrdqError) as e:
            trdq.qgemm_tiled(w, Xt, sx, Y)
        assert e.value.status == trdq.ERR_UNSUPPORTED
    for w in (w160, w4, w8):
        w.close()


def test_layer_takes_the_tiled_pair_for_large_shapes(oracle):
    """trdq_layer_forward with a workspace: shapes of more than one tile per compute unit go through the
    tiled pair (the workspace's layout is private to the layer); the result is the oracle's."""
    M, K, N = 4096, 256, 1152
    table = trdq.Table(4, 2)
    layer = trdq.Layer(table, K, N, 8)
    Xb, W, d, bias = wl.small_case(74, M, K, N)
    for g in range(2):
        layer.set_group(g, f32_to_dev(d), f32_to_dev(W))
    Xq_ws = torch.empty((M, K), dtype=torch.int8, device=dev())
    sx_ws = torch.empty((M,), dtype=torch.float32, device=dev())
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
    layer.forward(3, bf16_to_dev(Xb), Y, bias=f32_to_dev(bias), fused=False, Xq_ws=Xq_ws, sx_ws=sx_ws)
    torch.cuda.synchronize()
    ref = oracle.linear(Xb, W, d, bias, wbits=8, exact_blas=True)
    assert_y_close(bf16_to_host(Y), ref["Y"], "layer (tiled pair)")
    layer.close()
