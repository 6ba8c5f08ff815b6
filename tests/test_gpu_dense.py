"""GPU parity of the dense-block rotation path (the BlockDiag equation with arbitrary orthogonal
blocks, e.g. the greedy rotations of Eq. 6-7): trdq_rotation_create, trdq_rotate_quant_dense,
trdq_prepare_weights_dense and the unchanged product."""
import numpy as np
import pytest
import torch

from paper_2503_06564_amd import trdq, workloads as wl
from gpu_util import (assert_codes_close, assert_scales_close, assert_y_close, narrow_code_masks, bf16_to_dev, bf16_to_host,
                      dev, f32_to_dev)

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def _blocks(seed, K):
    """float32 orthogonal blocks [K/128, 128, 128] (non-symmetric)."""
    return wl.orthogonal_uniform_first_row(seed, K // 128).astype(np.float32)


def _rq_dense(Xbits, rot):
    M, K = Xbits.shape
    Xq = torch.full((M, K), 99, dtype=torch.int8, device=dev())
    sx = torch.full((M,), -1.0, dtype=torch.float32, device=dev())
    trdq.rotate_quant_dense(bf16_to_dev(Xbits), rot, Xq, sx)
    torch.cuda.synchronize()
    return Xq, sx


# a wave per block of a 16-token group, one and (from 8192 tokens on) two token tiles per piece load; rows wider
# than 12 blocks: a workgroup per block with its pieces in LDS, two passes
@pytest.mark.parametrize("M,K", [(1, 128), (37, 256), (300, 1152), (40, 2304), (64, 4608), (8200, 1152), (8200, 1664),
                                 (0, 256)])
def test_rotate_quant_dense_matches_oracle(oracle, M, K):
    say(f"rotate_quant_dense M={M} K={K}")
    Xb, _, d, _ = wl.small_case(61, max(M, 1), K, 16, n_outliers=max(1, K // 144), outlier=40.0)
    Xb = Xb[:M]
    Rs = _blocks(K, K)
    rot = trdq.Rotation(f32_to_dev(Rs.reshape(-1, 128)).view(-1, 128, 128), f32_to_dev(d))
    Xq, sx = _rq_dense(Xb, rot)
    if M:
        Xq_o, sx_o = oracle.quant_tokens(oracle.rotate_dense(Xb, d, Rs))
        assert_codes_close(Xq.cpu().numpy(), Xq_o, "Xq (dense blocks)")
        assert_scales_close(sx.cpu().numpy(), sx_o, "s_x (dense blocks)")
    rot.close()


def test_dense_path_with_hadamard_blocks_agrees_with_the_fast_path(oracle):
    M, K = 200, 1152
    Xb, _, d, _ = wl.small_case(62, M, K, 16, n_outliers=8)
    Hn = (oracle.hadamard(128).astype(np.float64) / np.sqrt(128.0)).astype(np.float32)
    Rs = np.stack([Hn] * (K // 128))
    rot = trdq.Rotation(f32_to_dev(Rs.reshape(-1, 128)).view(-1, 128, 128), f32_to_dev(d))
    Xq, sx = _rq_dense(Xb, rot)
    Xq2 = torch.empty_like(Xq); sx2 = torch.empty_like(sx)
    trdq.rotate_quant(bf16_to_dev(Xb), f32_to_dev(d), Xq2, sx2)
    torch.cuda.synchronize()
    # 1/sqrt(128) is not a float32 number: the dense blocks carry its rounding, codes may differ by one LSB rarely
    assert_codes_close(Xq.cpu().numpy(), Xq2.cpu().numpy(), "dense Hadamard blocks vs butterflies")
    assert_scales_close(sx.cpu().numpy(), sx2.cpu().numpy().astype(np.float64), "s_x")
    rot.close()


@pytest.mark.parametrize("M,K,N,wbits", [(17, 256, 144, 8), (300, 1152, 272, 8), (256, 1152, 288, 8), (64, 384, 160, 4),
                                         (130, 1152, 144, 6)])
def test_dense_linear_end_to_end(oracle, M, K, N, wbits):
    say(f"dense-block linear M={M} K={K} N={N} wbits={wbits}")
    Xb, W, d, bias = wl.small_case(63, M, K, N, n_outliers=max(1, K // 144), outlier=40.0)
    Rs = _blocks(7 + K, K)
    rot = trdq.Rotation(f32_to_dev(Rs.reshape(-1, 128)).view(-1, 128, 128), f32_to_dev(d))
    w = trdq.prepare_weights_dense(f32_to_dev(W), rot, wbits=wbits)
    ref = oracle.linear_dense(Xb, W, d, Rs, bias, wbits=wbits, exact_blas=True)
    codes, scales = w.export()
    assert_codes_close(codes, ref["Wq"], "Wq (dense blocks)")
    assert_scales_close(scales, ref["sw"], "s_w (dense blocks)")
    Xq, sx = _rq_dense(Xb, rot)
    assert_codes_close(Xq.cpu().numpy(), ref["Xq"], "Xq (dense blocks)")
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
    trdq.qgemm(w, Xq, sx, Y, bias=f32_to_dev(bias))
    torch.cuda.synchronize()
    assert_y_close(bf16_to_host(Y), ref["Y"], "Y (dense blocks)",
                   *narrow_code_masks(8, wbits, None, None, codes, ref["Wq"]))
    # the rotation cancels: close to the unquantised product as well
    exact = oracle.bf16_to_f64(Xb) @ W.astype(np.float64) + bias
    err = np.abs(oracle.bf16_to_f64(bf16_to_host(Y)) - exact).mean() / np.abs(exact).mean()
    assert err < {8: 0.04, 6: 0.12, 4: 0.4}[wbits], err
    w.close(); rot.close()


def test_greedy_blocks_from_the_oracle_run_on_the_gpu(oracle):
    # Eq. 6-7 on calibration activations (oracle), applied by the GPU path to fresh activations
    K, N, M = 256, 144, 96
    Xcal, W, d, bias = wl.small_case(64, 128, K, N, n_outliers=3, outlier=60.0)
    Qs = wl.orthogonal_uniform_first_row(9, 8)
    Rs, ns = oracle.greedy_rotations(Xcal, d, Qs)
    Rs32 = Rs.astype(np.float32)
    Xb = wl.small_case(65, M, K, N, n_outliers=0)[0]
    Xf = oracle.bf16_to_f64(Xb); Xf[:, :] += oracle.bf16_to_f64(Xcal[:M]) * 0.5       # same outlier channels
    Xb = wl.f32_to_bf16_bits(Xf.astype(np.float32))
    rot = trdq.Rotation(f32_to_dev(Rs32.reshape(-1, 128)).view(-1, 128, 128), f32_to_dev(d))
    Xq, sx = _rq_dense(Xb, rot)
    Xq_o, sx_o = oracle.quant_tokens(oracle.rotate_dense(Xb, d, Rs32))
    assert_codes_close(Xq.cpu().numpy(), Xq_o, "Xq (greedy blocks)")
    assert_scales_close(sx.cpu().numpy(), sx_o, "s_x (greedy blocks)")
    rot.close()


def test_dense_argument_errors():
    R = torch.zeros((2, 128, 128), device=dev())
    rot = trdq.Rotation(R)
    X = torch.zeros((4, 384), dtype=torch.bfloat16, device=dev())      # K of the input != K of the rotation
    Xq = torch.zeros((4, 384), dtype=torch.int8, device=dev())
    sx = torch.zeros((4,), device=dev())
    W = torch.zeros((384, 32), device=dev())
    with pytest.raises(trdq.TrdqError) as e:
        trdq.prepare_weights_dense(W, rot)
    assert e.value.status == trdq.ERR_MISMATCH
    rot.close()


@pytest.mark.parametrize("Mc,K,n_steps", [(128, 256, 8), (1000, 1152, 16), (37, 128, 1), (300, 384, 40)])
def test_greedy_rotation_matches_oracle(oracle, Mc, K, n_steps):
    say(f"greedy rotation Mc={Mc} K={K} steps={n_steps}")
    Xcal, _, d, _ = wl.small_case(66, Mc, K, 16, n_outliers=max(2, K // 100), outlier=60.0)
    Qs = wl.orthogonal_uniform_first_row(10, n_steps)
    R = torch.zeros((K // 128, 128, 128), dtype=torch.float32, device=dev())
    n = trdq.greedy_rotation(bf16_to_dev(Xcal), f32_to_dev(d), torch.from_numpy(Qs).to(dev()), R)
    torch.cuda.synchronize()
    Rs, ns = oracle.greedy_rotations(Xcal, d, Qs)
    assert np.array_equal(n, ns), (n, ns)
    Rg = R.cpu().numpy().astype(np.float64)
    assert np.abs(Rg - Rs).max() < 1e-6          # float64 on both sides, stored as float32
    for b in range(K // 128):
        assert np.abs(Rg[b] @ Rg[b].T - np.eye(128)).max() < 1e-5
    # and the blocks do what they are for: the largest rotated calibration activation is what the oracle says
    U = oracle.bf16_to_f64(Xcal) * d.astype(np.float64)
    for b in range(K // 128):
        got = np.abs(U[:, b * 128:(b + 1) * 128] @ Rg[b]).max()
        _, _, m = oracle.greedy_rotation(U[:, b * 128:(b + 1) * 128], Qs)
        assert abs(got - m[ns[b] - 1]) <= 1e-5 * m[ns[b] - 1]


def test_greedy_rotation_end_to_end_beats_no_rotation(oracle):
    # calibrate on one batch, run the rotated linear on another with the same outlier channels
    K, N, M = 384, 144, 200
    Xcal, W, d, bias = wl.small_case(67, 256, K, N, n_outliers=4, outlier=80.0)
    Qs = wl.orthogonal_uniform_first_row(11, 24)
    R = torch.zeros((K // 128, 128, 128), dtype=torch.float32, device=dev())
    trdq.greedy_rotation(bf16_to_dev(Xcal), f32_to_dev(d), torch.from_numpy(Qs).to(dev()), R)
    rot = trdq.Rotation(R, f32_to_dev(d))
    w = trdq.prepare_weights_dense(f32_to_dev(W), rot, wbits=8)
    Xf = oracle.bf16_to_f64(Xcal[:M]) * np.random.default_rng(3).uniform(0.5, 1.5, (M, 1))
    Xb = wl.f32_to_bf16_bits(Xf.astype(np.float32))
    Xq, sx = _rq_dense(Xb, rot)
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
    trdq.qgemm(w, Xq, sx, Y, bias=f32_to_dev(bias))
    torch.cuda.synchronize()
    ref = oracle.linear_dense(Xb, W, d, R.cpu().numpy(), bias, exact_blas=True)
    assert_codes_close(Xq.cpu().numpy(), ref["Xq"], "Xq (greedy blocks)")
    assert_codes_close(w.export()[0], ref["Wq"], "Wq (greedy blocks)")
    assert_y_close(bf16_to_host(Y), ref["Y"], "Y (greedy blocks)")
    exact = oracle.bf16_to_f64(Xb) @ W.astype(np.float64) + bias
    err_rot = np.abs(oracle.bf16_to_f64(bf16_to_host(Y)) - exact).mean()
    # the same W8A8 quantisers without any rotation (identity blocks) lose much more to the outliers
    eye = np.stack([np.eye(128, dtype=np.float32)] * (K // 128))
    err_plain = np.abs(oracle.linear_dense(Xb, W, d, eye, bias)["Yd"] - exact).mean()
    assert err_rot < 0.5 * err_plain, (err_rot, err_plain)
    w.close(); rot.close()


# ---- Eq. 10 in full with dense blocks: first rotation, permutation, second rotation ----

def _rot(Rs, d=None):
    return trdq.Rotation(f32_to_dev(Rs.reshape(-1, 128)).view(-1, 128, 128), None if d is None else f32_to_dev(d))


# K > 1536 takes the 8-token kernel: 13 blocks (waves with one and with two blocks), 18, 36; token counts around 8
@pytest.mark.parametrize("M,K", [(1, 128), (37, 256), (300, 1152), (64, 1536), (530, 384), (0, 256),
                                 (1, 1664), (40, 1664), (9, 2304), (70, 4608), (263, 4608)])
def test_rotate_quant_dense_rpr_matches_oracle(oracle, M, K):
    say(f"rotate_quant_dense_rpr M={M} K={K}")
    Xb, _, d, _ = wl.small_case(71, max(M, 1), K, 16, n_outliers=max(1, K // 144), outlier=40.0)
    Xb = Xb[:M]
    R1, R2 = _blocks(K + 1, K), _blocks(K + 2, K)
    perm = np.random.default_rng(K).permutation(K).astype(np.int32)
    rot1, rot2 = _rot(R1, d), _rot(R2)
    Xq = torch.full((M, K), 99, dtype=torch.int8, device=dev())
    sx = torch.full((M,), -1.0, dtype=torch.float32, device=dev())
    trdq.rotate_quant_dense_rpr(bf16_to_dev(Xb), rot1, torch.from_numpy(perm).to(dev()), rot2, Xq, sx)
    torch.cuda.synchronize()
    if M:
        Xq_o, sx_o = oracle.quant_tokens(oracle.rotate_dense_rpr(Xb, d, R1, perm, R2))
        assert_codes_close(Xq.cpu().numpy(), Xq_o, "Xq (dense R1 P R2)")
        assert_scales_close(sx.cpu().numpy(), sx_o, "s_x (dense R1 P R2)")
    rot1.close(); rot2.close()


# the workspace form: block-resident kernels around float32 once-rotated values (K > 1536, and narrower rows from
# 16384 tokens on); otherwise it is the plain call.  13 blocks and 36, token counts around the 16- and 32-token groups and beyond one round of workgroups.
# (from 8192 tokens on the second rotation takes two token tiles per fragment read)
@pytest.mark.parametrize("M,K", [(1, 1664), (40, 1664), (9, 2304), (33, 2304), (70, 4608), (263, 4608), (1100, 2304),
                                 (300, 1152), (0, 2304), (8230, 1664), (8192, 2304), (16400, 384), (16384, 128)])
def test_rotate_quant_dense_rpr_ws_matches_oracle(oracle, M, K):
    say(f"rotate_quant_dense_rpr_ws M={M} K={K}")
    Xb, _, d, _ = wl.small_case(74, max(M, 1), K, 16, n_outliers=max(1, K // 144), outlier=40.0)
    Xb = Xb[:M]
    R1, R2 = _blocks(K + 5, K), _blocks(K + 6, K)
    perm = np.random.default_rng(K + 1).permutation(K).astype(np.int32)
    rot1, rot2 = _rot(R1, d), _rot(R2)
    nbytes = trdq.rotate_quant_dense_rpr_ws_nbytes(M, K)
    assert (nbytes > 0) == (M > 0 and (K > 1536 or M >= 16384))
    ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device=dev()) if nbytes else None     # NaN patterns: nothing is read unwritten
    Xq = torch.full((M, K), 99, dtype=torch.int8, device=dev())
    sx = torch.full((M,), -1.0, dtype=torch.float32, device=dev())
    perm_dev = torch.from_numpy(perm).to(dev())
    for rep in range(2):        # the second call finds the first call's values in the workspace
        trdq.rotate_quant_dense_rpr_ws(bf16_to_dev(Xb), rot1, perm_dev, rot2, Xq, sx, ws)
    torch.cuda.synchronize()
    if M:
        Xq_o, sx_o = oracle.quant_tokens(oracle.rotate_dense_rpr(Xb, d, R1, perm, R2))
        assert_codes_close(Xq.cpu().numpy(), Xq_o, "Xq (dense R1 P R2, workspace form)")
        assert_scales_close(sx.cpu().numpy(), sx_o, "s_x (dense R1 P R2, workspace form)")
    rot1.close(); rot2.close()


def test_dense_rpr_ws_argument_errors():
    K = 2304
    R = torch.zeros((K // 128, 128, 128), device=dev())
    rot1, rot2 = trdq.Rotation(R, torch.ones((K,), device=dev())), trdq.Rotation(R)
    X = torch.zeros((40, K), dtype=torch.bfloat16, device=dev())
    Xq = torch.zeros((40, K), dtype=torch.int8, device=dev())
    sx = torch.zeros((40,), device=dev())
    perm = torch.arange(K, dtype=torch.int32, device=dev())
    need = trdq.rotate_quant_dense_rpr_ws_nbytes(40, K)
    with pytest.raises(trdq.TrdqError) as e:
        trdq.rotate_quant_dense_rpr_ws(X, rot1, perm, rot2, Xq, sx, None)
    assert e.value.status == trdq.ERR_NULL
    with pytest.raises(trdq.TrdqError) as e:
        trdq.rotate_quant_dense_rpr_ws(X, rot1, perm, rot2, Xq, sx, torch.empty((need - 4,), dtype=torch.uint8, device=dev()))
    assert e.value.status == trdq.ERR_SHAPE
    ws = torch.empty((need + 16,), dtype=torch.uint8, device=dev())
    with pytest.raises(trdq.TrdqError) as e:
        trdq.rotate_quant_dense_rpr_ws(X, rot1, perm, rot2, Xq, sx, ws[4:])         # not 16-byte aligned
    assert e.value.status == trdq.ERR_SHAPE
    rot1.close(); rot2.close()


@pytest.mark.parametrize("M,K,N,wbits", [(17, 256, 144, 8), (300, 1152, 272, 8), (64, 384, 160, 4), (50, 4608, 144, 8)])
def test_dense_rpr_linear_end_to_end(oracle, M, K, N, wbits):
    say(f"dense R1 P R2 linear M={M} K={K} N={N} wbits={wbits}")
    Xb, W, d, bias = wl.small_case(72, M, K, N, n_outliers=max(1, K // 144), outlier=40.0)
    R1, R2 = _blocks(K + 3, K), _blocks(K + 4, K)
    perm = oracle.zigzag(np.abs(oracle.rotate_dense(Xb, d, R1)).max(axis=0), 128).astype(np.int32)
    rot1, rot2 = _rot(R1, d), _rot(R2)
    perm_dev = torch.from_numpy(perm).to(dev())
    w = trdq.prepare_weights_dense_rpr(f32_to_dev(W), rot1, perm_dev, rot2, wbits=wbits)
    ref = oracle.linear_dense_rpr(Xb, W, d, R1, perm, R2, bias, wbits=wbits, exact_blas=True)
    codes, scales = w.export()
    assert_codes_close(codes, ref["Wq"], "Wq (dense R1 P R2)")
    assert_scales_close(scales, ref["sw"], "s_w (dense R1 P R2)")
    Xq = torch.empty((M, K), dtype=torch.int8, device=dev())
    sx = torch.empty((M,), dtype=torch.float32, device=dev())
    trdq.rotate_quant_dense_rpr(bf16_to_dev(Xb), rot1, perm_dev, rot2, Xq, sx)
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
    trdq.qgemm(w, Xq, sx, Y, bias=f32_to_dev(bias))
    torch.cuda.synchronize()
    assert_codes_close(Xq.cpu().numpy(), ref["Xq"], "Xq (dense R1 P R2)")
    assert_y_close(bf16_to_host(Y), ref["Y"], "Y (dense R1 P R2)")
    w.close(); rot1.close(); rot2.close()


def test_dense_rpr_argument_errors():
    R = torch.zeros((2, 128, 128), device=dev())
    d = torch.ones((256,), device=dev())
    rot1, rot2_bad, rot2 = trdq.Rotation(R, d), trdq.Rotation(R, d), trdq.Rotation(R)
    X = torch.zeros((4, 256), dtype=torch.bfloat16, device=dev())
    Xq = torch.zeros((4, 256), dtype=torch.int8, device=dev())
    sx = torch.zeros((4,), device=dev())
    perm = torch.arange(256, dtype=torch.int32, device=dev())
    with pytest.raises(trdq.TrdqError) as e:
        trdq.rotate_quant_dense_rpr(X, rot1, perm, rot2_bad, Xq, sx)      # the second rotation carries a diagonal
    assert e.value.status == trdq.ERR_MISMATCH
    with pytest.raises(trdq.TrdqError) as e:
        trdq.Rotation(torch.zeros((37, 128, 128), device=dev()))          # more than 36 blocks: no kernel takes them
    assert e.value.status == trdq.ERR_UNSUPPORTED
    for r in (rot1, rot2_bad, rot2):
        r.close()


@pytest.mark.parametrize("Mc,K,steps", [(128, 256, 6), (500, 1152, 10)])
def test_time_rotation_calibration_chain(oracle, Mc, K, steps):
    """Sec. 3.2 end to end on the GPU: greedy R1, channel maxima after it, zigzag P, greedy R2 on the
    rotated and permuted activations; every stage against the oracle, then the rotated linear."""
    say(f"calibration chain Mc={Mc} K={K} steps={steps}")
    N = 144
    Xcal, W, d, bias = wl.small_case(73, Mc, K, N, n_outliers=max(2, K // 100), outlier=60.0)
    Q1 = wl.orthogonal_uniform_first_row(12, steps)
    Q2 = wl.orthogonal_uniform_first_row(13, steps)
    X = bf16_to_dev(Xcal)
    dd = f32_to_dev(d)
    nb = K // 128
    # first rotation
    R1 = torch.zeros((nb, 128, 128), dtype=torch.float32, device=dev())
    n1 = trdq.greedy_rotation(X, dd, torch.from_numpy(Q1).to(dev()), R1)
    R1_o, n1_o = oracle.greedy_rotations(Xcal, d, Q1)
    assert np.array_equal(n1, n1_o) and np.abs(R1.cpu().numpy() - R1_o).max() < 1e-6
    rot1 = trdq.Rotation(R1, dd)
    R1h = R1.cpu().numpy()
    # channel maxima after it, permutation
    mag = torch.full((K,), -1.0, dtype=torch.float32, device=dev())
    trdq.channel_absmax_dense(X, rot1, mag)
    torch.cuda.synchronize()
    V1 = oracle.rotate_dense(Xcal, d, R1h)
    assert np.allclose(mag.cpu().numpy(), np.abs(V1).max(axis=0), rtol=1e-5, atol=0)
    perm = trdq.zigzag_permutation(mag.cpu().numpy())
    assert np.array_equal(perm, oracle.zigzag(mag.cpu().numpy().astype(np.float64), 128))
    perm_dev = torch.from_numpy(perm).to(dev())
    # second rotation on the rotated, permuted activations
    R2 = torch.zeros((nb, 128, 128), dtype=torch.float32, device=dev())
    n2 = trdq.greedy_rotation_second(X, rot1, perm_dev, torch.from_numpy(Q2).to(dev()), R2)
    V2 = V1[:, perm.astype(np.int64)]
    for b in range(nb):
        R2_o, n2_o, _ = oracle.greedy_rotation(V2[:, b * 128:(b + 1) * 128], Q2)
        assert n2[b] == n2_o and np.abs(R2[b].cpu().numpy() - R2_o).max() < 1e-6
    rot2 = trdq.Rotation(R2)
    # the rotated linear with what was calibrated
    M = min(Mc, 96)
    Xb = Xcal[:M]
    w = trdq.prepare_weights_dense_rpr(f32_to_dev(W), rot1, perm_dev, rot2)
    Xq = torch.empty((M, K), dtype=torch.int8, device=dev())
    sx = torch.empty((M,), dtype=torch.float32, device=dev())
    trdq.rotate_quant_dense_rpr(bf16_to_dev(Xb), rot1, perm_dev, rot2, Xq, sx)
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
    trdq.qgemm(w, Xq, sx, Y, bias=f32_to_dev(bias))
    torch.cuda.synchronize()
    ref = oracle.linear_dense_rpr(Xb, W, d, R1h, perm, R2.cpu().numpy(), bias, exact_blas=True)
    assert_codes_close(Xq.cpu().numpy(), ref["Xq"], "Xq (calibrated R1 P R2)")
    assert_codes_close(w.export()[0], ref["Wq"], "Wq (calibrated R1 P R2)")
    assert_y_close(bf16_to_host(Y), ref["Y"], "Y (calibrated R1 P R2)")
    exact = oracle.bf16_to_f64(Xb) @ W.astype(np.float64) + bias
    err = np.abs(oracle.bf16_to_f64(bf16_to_host(Y)) - exact).mean()
    eye = np.stack([np.eye(128, dtype=np.float32)] * nb)
    err_plain = np.abs(oracle.linear_dense(Xb, W, d, eye, bias)["Yd"] - exact).mean()
    assert err < 0.5 * err_plain, (err, err_plain)
    w.close(); rot1.close(); rot2.close()
