"""Helpers of the GPU parity tests: device marshalling and the tolerance checks.

Tolerances (stated by the benchmark spec, derived in the design notes):
  codes     identical except <= 1 LSB on <= 0.01 % of elements (fp32 vs fp64 rotation at ties)
  int32 acc bit-exact given identical codes
  scales    rtol 1e-5
  bf16 Y    within 1e-2 x row absmax of the oracle's quantised output
"""
import numpy as np
import torch

from paper_2503_06564_amd import trdq

CODE_FRAC = 1e-4
SCALE_RTOL = 1e-5
Y_TOL = 1e-2


def dev():
    return torch.device("cuda:0")


def bf16_to_dev(bits):
    """uint16 bf16 bit patterns [.., ..] -> torch.bfloat16 tensor on the GPU."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev())
    return t.view(torch.bfloat16)


def bf16_to_host(t):
    """torch.bfloat16 tensor -> uint16 bit patterns (numpy)."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def f32_to_dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev())


def bits_to_f64(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def gpu_rotate_quant(Xbits, d, ldx=None):
    M, K = Xbits.shape
    if ldx is None:
        X = bf16_to_dev(Xbits)
    else:
        buf = torch.zeros((max(M, 1), ldx), dtype=torch.bfloat16, device=dev())
        X = buf[:M, :K]
        X.copy_(bf16_to_dev(Xbits))
    Xq = torch.full((M, K), 99, dtype=torch.int8, device=dev())
    sx = torch.full((M,), -1.0, dtype=torch.float32, device=dev())
    trdq.rotate_quant(X, f32_to_dev(d), Xq, sx)
    torch.cuda.synchronize()
    return Xq, sx


def gpu_qgemm(w, Xq, sx, bias, N, debug=True, ldy=None):
    M = Xq.shape[0]
    K, _, wbits = w.info()
    if ldy is None:
        Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
    else:
        Y = torch.zeros((max(M, 1), ldy), dtype=torch.bfloat16, device=dev())[:M, :N]
    acc = None
    if debug:
        shape = (M, N) if wbits == 8 else (K // 128, M, N)
        acc = torch.full(shape, -7, dtype=torch.int32, device=dev())
    trdq.qgemm(w, Xq, sx, Y, bias=f32_to_dev(bias), acc_debug=acc)
    torch.cuda.synchronize()
    return Y, acc


def assert_codes_close(got, want, what):
    got = np.asarray(got, dtype=np.int16)
    want = np.asarray(want, dtype=np.int16)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    diff = np.abs(got - want)
    n_bad = int(np.count_nonzero(diff))
    assert diff.max(initial=0) <= 1, f"{what}: code differs by {diff.max()} LSB"
    assert n_bad <= CODE_FRAC * diff.size, f"{what}: {n_bad} of {diff.size} codes differ (> 0.01 %)"
    return n_bad


def assert_scales_close(got, want, what):
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.allclose(got, want, rtol=SCALE_RTOL, atol=0), \
        f"{what}: max rel err {np.max(np.abs(got - want) / np.maximum(np.abs(want), 1e-300))}"


def assert_y_close(got_bits, want_bits, what, skip_rows=None, skip_cols=None):
    """|got - want| <= 1e-2 x row absmax of want, element by element.

    skip_rows / skip_cols: boolean masks of tokens / output channels whose activation / weight
    codes legitimately differ from the oracle's by one LSB (the <= 0.01 % allowance).  One such
    step moves the affected outputs by s_x * s_w * |other code|, which for int4 weights can
    exceed 1e-2 x row absmax, so those entries are judged on identical codes instead (the
    caller compares them with the oracle's epilogue run on the GPU's own codes)."""
    got, want = bits_to_f64(got_bits), bits_to_f64(want_bits)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if got.size == 0:
        return 0.0
    row = np.abs(want).max(axis=1, keepdims=True)
    err = np.abs(got - want)
    ok = err <= Y_TOL * row + 1e-30
    if skip_rows is not None:
        ok = ok | np.asarray(skip_rows, bool)[:, None]
    if skip_cols is not None:
        ok = ok | np.asarray(skip_cols, bool)[None, :]
    worst = float((np.where(ok, 0.0, err) / np.maximum(row, 1e-30)).max())
    assert np.all(ok), f"{what}: max err / row absmax = {worst}"
    return float((err / np.maximum(row, 1e-30)).max())
