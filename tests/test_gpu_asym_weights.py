"""GPU parity of asymmetric per-output-channel weights (Eq. 1-3 applied to H_t(W)): trdq_prepare_weights_asym,
trdq_weights_export_zero_points and trdq_qgemm_asym_weights against the oracle, with symmetric and with
asymmetric activation codes."""
import numpy as np
import pytest
import torch

from paper_2503_06564_amd import trdq, workloads as wl
from gpu_util import (CODE_FRAC, assert_asym_codes_close, assert_codes_close, assert_scales_close, assert_y_close,
                      assert_y_same_codes, bf16_to_dev, bf16_to_host, dev, f32_to_dev)

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def _weights(oracle, W, d):
    """GPU weight set and its (unsigned codes, scales, zero points) checked against the oracle's."""
    w = trdq.prepare_weights_asym(f32_to_dev(W), f32_to_dev(d))
    stored, scales = w.export()
    zw = trdq.weights_zero_points(w)
    q = stored.astype(np.int16) + 128
    Wq_o, sw_o, zw_o = oracle.prepare_weights_asym(W, d, 128, 8)
    assert q.min() >= 0 and q.max() <= 255
    # a zero point is -rint(lo / s) with |lo / s| <= 255: fp32 against float64 may move it across a tie on a rare
    # channel; its codes move with it and the reconstruction s (q - z) does not, so q - z is what is compared
    dz = np.abs(zw - zw_o)
    assert dz.max(initial=0) <= 1 and np.count_nonzero(dz) <= max(1, len(zw) // 1000)
    diff = np.abs((q - zw[None, :]) - (Wq_o.astype(np.int16) - zw_o[None, :]))
    assert diff.max(initial=0) <= 1
    assert np.count_nonzero(diff) <= CODE_FRAC * diff.size + 2 * np.count_nonzero(dz)
    assert_scales_close(scales, sw_o, "s_w (asymmetric)")
    return w, q.astype(np.uint8), scales, zw


@pytest.mark.parametrize("K,N", [(128, 16), (256, 48), (1152, 1152), (4608, 80), (384, 208)])
def test_prepare_weights_asym_matches_oracle(oracle, K, N):
    say(f"prepare_weights_asym K={K} N={N}")
    _, W, d, _ = wl.small_case(81, 4, K, N)
    W += np.float32(0.01) * np.random.default_rng(K + N).standard_normal((1, N)).astype(np.float32)   # skewed channels
    W[:, N // 2] = 0.0                               # a dead channel
    W[:, 1] = np.abs(W[:, 1])                        # (rotation mixes signs: stays two-sided after it)
    w, q, scales, zw = _weights(oracle, W, d)
    assert w.info() == (K, N, 8)
    assert scales[N // 2] == 0 and zw[N // 2] == 0 and not q[:, N // 2].any()
    live = scales > 0
    assert np.all(q[:, live].min(axis=0) == 0) or np.all(q[:, live].max(axis=0) == 255)
    w.close()


@pytest.mark.parametrize("M,K,N", [(1, 128, 16), (17, 256, 144), (300, 4608, 272), (513, 384, 400), (1024, 1152, 1152),
                                   (4100, 512, 1152)])
@pytest.mark.parametrize("act_asym", [False, True])
def test_linear_asym_weights_end_to_end(oracle, M, K, N, act_asym):
    say(f"linear, asymmetric weights M={M} K={K} N={N} act_asym={act_asym}")
    Xb, W, d, bias = wl.small_case(82, M, K, N, n_outliers=max(1, K // 144), outlier=40.0)
    W += np.float32(0.01) * np.random.default_rng(7).standard_normal((1, N)).astype(np.float32)
    w, q_w, scales, zw = _weights(oracle, W, d)
    X, dd = bf16_to_dev(Xb), f32_to_dev(d)
    Xq = torch.empty((M, K), dtype=torch.int8, device=dev())
    sx = torch.empty((M,), dtype=torch.float32, device=dev())
    zc = torch.empty((M,), dtype=torch.int32, device=dev()) if act_asym else None
    if act_asym:
        trdq.rotate_quant_asym(X, dd, Xq, sx, zc, warm=w)
    else:
        trdq.rotate_quant(X, dd, Xq, sx, warm=w)
    rowsum = torch.full((M,), -5, dtype=torch.int32, device=dev())
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
    acc = torch.full((M, N), -7, dtype=torch.int32, device=dev())
    trdq.qgemm_asym_weights(w, Xq, sx, zc, rowsum, Y, bias=f32_to_dev(bias), acc_debug=acc)
    torch.cuda.synchronize()
    ref = oracle.linear_asym_weights(Xb, W, d, bias, exact_blas=True, act_asym=act_asym)
    if act_asym:
        qx = Xq.cpu().numpy().astype(np.int16) + 128
        zx = (128 - zc.cpu().numpy()).astype(np.int32)
        assert_asym_codes_close(qx, zx, ref["Xq"], ref["zx"], "Xq (asymmetric)")
    else:
        qx, zx = Xq.cpu().numpy().astype(np.int16), None
        assert_codes_close(qx, ref["Xq"], "Xq")
    assert np.array_equal(rowsum.cpu().numpy(), Xq.cpu().numpy().astype(np.int64).sum(axis=1))
    # integer sums bit-exact on the GPU's own codes and zero points
    want_acc = oracle.acc_asym2_exact_blas(qx, zx, q_w, zw)
    assert np.array_equal(acc.cpu().numpy(), want_acc), "integer sums differ on the GPU's own codes"
    y_same = oracle.dequant(want_acc, sx.cpu().numpy(), scales, bias)
    assert_y_same_codes(bf16_to_host(Y), y_same, "Y (same codes)")
    assert_y_close(bf16_to_host(Y), ref["Y"], "Y (oracle end to end)")
    Y2 = torch.zeros_like(Y)
    trdq.qgemm_asym_weights(w, Xq, sx, zc, rowsum, Y2, bias=f32_to_dev(bias))
    torch.cuda.synchronize()
    assert torch.equal(Y2, Y)
    w.close()


def test_asym_weights_are_refused_by_the_other_products(oracle):
    M, K, N = 128, 256, 144
    Xb, W, d, _ = wl.small_case(83, M, K, N)
    wa = trdq.prepare_weights_asym(f32_to_dev(W), f32_to_dev(d))
    ws = trdq.prepare_weights(f32_to_dev(W), f32_to_dev(d))
    Xq = torch.zeros((M, K), dtype=torch.int8, device=dev())
    sx = torch.ones((M,), dtype=torch.float32, device=dev())
    zc = torch.zeros((M,), dtype=torch.int32, device=dev())
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
    for call in (lambda: trdq.qgemm(wa, Xq, sx, Y), lambda: trdq.qgemm_asym(wa, Xq, sx, zc, Y),
                 lambda: trdq.linear_fused(bf16_to_dev(Xb), f32_to_dev(d), wa, Y),
                 lambda: trdq.qgemm_asym_weights(ws, Xq, sx, None, zc, Y)):
        with pytest.raises(trdq.TrdqError) as e:
            call()
        assert e.value.status == trdq.ERR_MISMATCH
    assert not trdq.qgemm_tiled_supported(wa, M)
    with pytest.raises(trdq.TrdqError) as e:
        trdq.weights_zero_points(ws)
    assert e.value.status == trdq.ERR_MISMATCH
    wa.close(); ws.close()
