"""Pins of the CPU oracle against what the paper and the mathematics fix.

Each test checks an oracle function against something that is not the oracle:
integer identities, a library routine (scipy's Sylvester construction, a float64
BLAS product, torch's float32->bfloat16 cast), closed forms, exact rational
brute force on tiny inputs, and the computational-invariance identity of
Eq. 4 / Eq. 9 / Eq. 10.  None needs a GPU.
"""
from fractions import Fraction

import numpy as np
import pytest
import scipy.linalg

from paper_2503_06564_amd import workloads as wl


# ----------------------------------------------------------------- Hadamard

@pytest.mark.parametrize("B", [2, 8, 128])
def test_hadamard_orthogonal_integer_exact(oracle, B):
    # R R^T = I per block (orthogonal rotation, Sec. 3.2): H H^T = B I in integers
    H = oracle.hadamard(B).astype(np.int64)
    assert set(np.unique(H)) == {-1, 1}
    assert np.array_equal(H @ H.T, B * np.eye(B, dtype=np.int64))
    assert np.array_equal(H, H.T)


@pytest.mark.parametrize("B", [8, 128])
def test_hadamard_is_sylvester(oracle, B):
    H = oracle.hadamard(B)
    assert np.array_equal(H, scipy.linalg.hadamard(B).astype(np.int8))
    h = B // 2
    assert np.array_equal(H[:h, :h], H[:h, h:])
    assert np.array_equal(H[:h, :h], H[h:, :h])
    assert np.array_equal(H[:h, :h], -H[h:, h:])


# ----------------------------------------------------------------- rotation

def _bf16(x):
    return wl.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_rotate_unit_vectors_give_hadamard_rows(oracle):
    B, K = 128, 256
    X = np.zeros((K, K), dtype=np.float32)
    X[np.arange(K), np.arange(K)] = 1.0
    V = oracle.rotate(_bf16(X), None, B)
    H = scipy.linalg.hadamard(B) / np.sqrt(B)
    expect = np.zeros((K, K))
    expect[:B, :B] = H
    expect[B:, B:] = H                     # block diagonal: no leakage across blocks
    assert np.allclose(V, expect, rtol=0, atol=1e-15)
    Xq, sx = oracle.quant_tokens(V)
    nz = expect != 0
    assert np.all(np.abs(Xq[nz]) == 127) and np.all(Xq[~nz] == 0)
    assert np.array_equal(np.sign(Xq[nz]), np.sign(expect[nz]).astype(np.int8))
    assert np.allclose(sx, 1 / np.sqrt(B) / 127, rtol=1e-15)


def test_rotate_constant_block_concentrates(oracle):
    B = 128
    X = np.concatenate([np.full((1, B), 0.5), np.full((1, B), -2.0)], axis=1).astype(np.float32)
    V = oracle.rotate(_bf16(X), None, B)[0]
    expect = np.zeros(2 * B)
    expect[0] = 0.5 * np.sqrt(B)
    expect[B] = -2.0 * np.sqrt(B)
    assert np.allclose(V, expect, rtol=0, atol=1e-13)


def test_rotate_applies_diag_as_multiplier_per_channel(oracle):
    # (X . Delta) R of Eq. 9/10: channel k is multiplied by d[k] before the rotation
    B, K = 8, 16
    r = np.random.default_rng(1)
    d = r.uniform(0.5, 2.0, K).astype(np.float32)
    X = np.zeros((K, K), dtype=np.float32)
    X[np.arange(K), np.arange(K)] = 1.0
    V = oracle.rotate(_bf16(X), d, B)
    H = scipy.linalg.hadamard(B) / np.sqrt(B)
    for k in range(K):
        b = k // B
        expect = np.zeros(K)
        expect[b * B:(b + 1) * B] = float(d[k]) * H[k % B]
        assert np.allclose(V[k], expect, rtol=1e-15, atol=0)


def test_rotate_preserves_row_norm(oracle):
    cfg = wl.CONFIGS[0]
    X = wl.make_x(cfg, "proj", M=64)
    d = wl.make_diag(wl.CONFIGS[1], "proj", 3)
    V = oracle.rotate(X, d)
    U = wl.bf16_bits_to_f32(X).astype(np.float64) * d.astype(np.float64)
    assert np.allclose(np.linalg.norm(V, axis=1), np.linalg.norm(U, axis=1), rtol=1e-12)


def test_rotation_narrows_outlier_rows(oracle):
    # Fig. 1 of the paper: the rotated activations have a much smaller range
    cfg = wl.CONFIGS[0]
    X = wl.make_x(cfg, "proj", M=128)
    V = oracle.rotate(X)
    before = np.abs(wl.bf16_bits_to_f32(X)).max(axis=1)
    after = np.abs(V).max(axis=1)
    assert np.median(before / after) > 3.0


@pytest.mark.parametrize("B,K,N,M", [(8, 24, 5, 7), (128, 256, 96, 33)])
def test_computational_invariance(oracle, B, K, N, M):
    # (X D R)(R^T D^-1 W) = X W, Eq. 9 / Eq. 10, unquantised, float64, to 1e-9
    Xb, W, d, _ = wl.small_case(5, M, K, N)
    V = oracle.rotate(Xb, d, B)
    Wp = oracle.rotate_weights(W, d, B)
    exact = wl.bf16_bits_to_f32(Xb).astype(np.float64) @ W.astype(np.float64)
    err = np.abs(V @ Wp - exact).max() / np.abs(exact).max()
    assert err < 1e-9
    # and the weight side really uses 1/d and the transpose: a wrong direction breaks it
    Wp_bad = oracle.rotate_weights(W, (1.0 / d).astype(np.float32), B)
    assert np.abs(V @ Wp_bad - exact).max() / np.abs(exact).max() > 1e-3


def test_rotate_weights_matches_dense_blockdiag(oracle):
    B, K, N = 8, 24, 6
    _, W, d, _ = wl.small_case(6, 4, K, N)
    R = np.kron(np.eye(K // B), scipy.linalg.hadamard(B) / np.sqrt(B))
    expect = R.T @ np.diag(1.0 / d.astype(np.float64)) @ W.astype(np.float64)
    assert np.allclose(oracle.rotate_weights(W, d, B), expect, rtol=1e-13, atol=1e-16)


# ---------------------------------------------------------------- quantiser

def test_quant_tokens_properties(oracle):
    cfg = wl.CONFIGS[0]
    V = oracle.rotate(wl.make_x(cfg, "proj", M=96))
    V[5] = 0.0                                            # a dead token
    Xq, sx = oracle.quant_tokens(V)
    live = np.ones(len(V), bool); live[5] = False
    assert np.all(np.abs(Xq[live]).max(axis=1) == 127)    # extreme value maps to +-127
    assert np.all(np.abs(Xq) <= 127)
    assert np.allclose(sx[live], np.abs(V[live]).max(axis=1) / 127, rtol=1e-15)
    assert sx[5] == 0 and np.all(Xq[5] == 0)
    # nearest rounding: reconstruction error at most half a step (Eq. 1)
    assert np.all(np.abs(V - sx[:, None] * Xq) <= sx[:, None] * (0.5 + 1e-12))
    # idempotent on its own grid
    Xq2, sx2 = oracle.quant_tokens(sx[:, None] * Xq)
    assert np.array_equal(Xq2, Xq) and np.allclose(sx2, sx, rtol=1e-15)


def test_quant_tokens_ties_to_even_and_sign(oracle):
    # row absmax 127 -> scale exactly 1; halves must go to the even neighbour
    V = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.49, -126.5, 126.5]])
    Xq, sx = oracle.quant_tokens(V)
    assert sx[0] == 1.0
    assert Xq[0].tolist() == [127, 0, 2, 2, 0, -2, -2, 3, -126, 126]


@pytest.mark.parametrize("wbits,qmax", [(8, 127), (4, 7)])
def test_quant_weights_properties(oracle, wbits, qmax):
    B, K, N = 128, 384, 40
    _, W, d, _ = wl.small_case(7, 4, K, N)
    Wp = oracle.rotate_weights(W, d, B)
    Wp[:, 3] = 0.0                                        # a dead output channel
    Wq, sw = oracle.quant_weights(Wp, wbits, B)
    assert np.abs(Wq).max() == qmax and np.all(np.abs(Wq) <= qmax)
    if wbits == 8:
        assert sw.shape == (N,)
        assert np.allclose(sw, np.abs(Wp).max(axis=0) / 127, rtol=1e-15)   # per output channel
        s_full = np.broadcast_to(sw, (K, N))
        assert np.all(np.abs(Wq[:, np.arange(N) != 3]).max(axis=0) == 127)
    else:
        assert sw.shape == (K // B, N)
        expect = np.abs(Wp.reshape(K // B, B, N)).max(axis=1) / 7          # per 128-row group
        assert np.allclose(sw, expect, rtol=1e-15)
        s_full = np.repeat(sw, B, axis=0)
    assert np.all(sw[..., 3] == 0) and np.all(Wq[:, 3] == 0)
    assert np.all(np.abs(Wp - s_full * Wq) <= s_full * (0.5 + 1e-12))


def test_int4_pack_layout_and_roundtrip(oracle):
    K, N = 6, 3
    Wq = np.array([[1, -1, 7], [-7, 0, 2], [3, 3, 3], [-3, -4, 5], [0, 0, 0], [-1, 6, -6]], dtype=np.int8)
    P = oracle.pack_int4(Wq)
    assert P.shape == (K // 2, N)
    # low nibble = even k, high nibble = odd k, two's complement
    assert P[0, 0] == (1 | (0x9 << 4))          # k=0: 1, k=1: -7 -> 0x9
    assert P[0, 1] == (0xF | (0x0 << 4))        # -1 -> 0xF
    assert P[2, 2] == (0x0 | (0xA << 4))        # -6 -> 0xA
    assert np.array_equal(oracle.unpack_int4(P), Wq)
    r = np.random.default_rng(0).integers(-7, 8, size=(256, 17)).astype(np.int8)
    assert np.array_equal(oracle.unpack_int4(oracle.pack_int4(r)), r)


# ------------------------------------------------------------ integer product

def test_igemm_brute_force_4x8x8(oracle):
    r = np.random.default_rng(3)
    Xq = r.integers(-127, 128, size=(4, 8)).astype(np.int8)
    Wq = r.integers(-127, 128, size=(8, 8)).astype(np.int8)
    acc = oracle.igemm(Xq, Wq)
    for i in range(4):
        for n in range(8):
            assert acc[i, n] == sum(int(Xq[i, k]) * int(Wq[k, n]) for k in range(8))
    accg = oracle.igemm(Xq, Wq, group=4)
    assert accg.shape == (2, 4, 8)
    for g in range(2):
        for i in range(4):
            for n in range(8):
                assert accg[g, i, n] == sum(int(Xq[i, k]) * int(Wq[k, n]) for k in range(4 * g, 4 * g + 4))


def test_igemm_equals_exact_float64_blas(oracle):
    r = np.random.default_rng(4)
    M, K, N = 37, 1152, 53                     # non-square: a transposed operand cannot pass
    Xq = r.integers(-127, 128, size=(M, K)).astype(np.int8)
    Wq = r.integers(-127, 128, size=(K, N)).astype(np.int8)
    Xq[0, :] = 127; Wq[:, 0] = 127             # the largest possible accumulator
    acc = oracle.igemm(Xq, Wq)
    assert acc[0, 0] == 127 * 127 * K
    assert np.array_equal(acc, (Xq.astype(np.float64) @ Wq.astype(np.float64)).astype(np.int64))
    assert np.array_equal(acc, oracle.acc_exact_blas(Xq, Wq))
    accg = oracle.igemm(Xq, Wq, group=128)
    assert np.array_equal(accg, oracle.acc_exact_blas(Xq, Wq, group=128))
    assert np.array_equal(accg.sum(axis=0), acc)


# ------------------------------------------------------------------ bf16 cast

def test_f64_to_bf16_matches_torch_on_float32_inputs(oracle):
    import torch
    r = np.random.default_rng(8)
    x = np.concatenate([
        r.standard_normal(4000).astype(np.float32) * np.float32(10.0) ** r.integers(-30, 30, 4000).astype(np.float32),
        np.array([0.0, -0.0, 1.0, -1.0, 3.3895314e38, -3.3895314e38, 1e-40, -1e-45, 65504.0], np.float32),
    ])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.f64_to_bf16(x.astype(np.float64))
    assert np.array_equal(got, want)
    assert np.array_equal(oracle.bf16_to_f64(got), wl.bf16_bits_to_f32(got).astype(np.float64))


def test_f64_to_bf16_rounds_once(oracle):
    # values where float64 -> float32 -> bf16 would round twice and land elsewhere
    cases = {
        1.0 + 2.0 ** -8 + 2.0 ** -30: 0x3F81,      # just above a tie: up
        1.0 + 2.0 ** -8 - 2.0 ** -30: 0x3F80,      # just below a tie: down
        1.0 + 2.0 ** -8: 0x3F80,                   # exact tie: to even (down)
        1.0 + 3 * 2.0 ** -8: 0x3F82,               # exact tie: to even (up)
        -(1.0 + 2.0 ** -8 + 2.0 ** -30): 0xBF81,
        3.4e38: 0x7F80,                            # above the largest bf16 + half step: inf
    }
    for y, bits in cases.items():
        assert int(oracle.f64_to_bf16(np.array([y]))[0]) == bits, y


# ------------------------------------------------------------------- dequant

def test_dequant_closed_form(oracle):
    acc = np.array([[100, -200, 0], [1, 2, 3]], dtype=np.int32)
    sx = np.array([0.5, 2.0]); sw = np.array([0.25, 1.0, 4.0])
    bias = np.array([1.0, 0.0, -3.0], dtype=np.float32)
    Y, Yd = oracle.dequant(acc, sx, sw, bias, return_f64=True)
    expect = np.array([[100 * .5 * .25 + 1, -200 * .5, -3.0], [1 * 2 * .25 + 1, 4.0, 3 * 2 * 4 - 3.0]])
    assert np.array_equal(Yd, expect)                      # all exactly representable
    assert np.array_equal(wl.bf16_bits_to_f32(Y), expect.astype(np.float32))
    # grouped form: s_x * sum_g s_w[g] acc[g] + bias
    accg = np.stack([acc, 2 * acc]); swg = np.stack([sw, 0.5 * sw])
    _, Ydg = oracle.dequant(accg, sx, swg, None, return_f64=True)
    assert np.array_equal(Ydg, 2 * (expect - bias))


# ---------------------------------------------------- whole path, tiny + exact

def _round_half_even_fraction(q):
    f = q.numerator // q.denominator           # floor
    rem = q - f
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and f % 2):
        f += 1
    return f


def _brute_force_codes(vals):
    """codes of one quantisation group from exact rationals: rint(127 v / max|v|)."""
    a = max(abs(v) for v in vals)
    return [0 if a == 0 else _round_half_even_fraction(v * 127 / a) for v in vals]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_whole_path_brute_force_4x8x8(oracle, seed):
    """M=4, K=8, N=8, B=8, W8A8, every step redone in exact rational arithmetic.

    The codes depend only on ratios inside a row/column, so the irrational 1/sqrt(B)
    cancels and the unnormalised Hadamard sums decide them exactly."""
    M = K = N = B = 8
    M = 4
    Xb, W, d, bias = wl.small_case(seed, M, K, N, n_outliers=1, outlier=20.0)
    out = oracle.linear(Xb, W, d, bias, B=B, wbits=8)
    X = [[Fraction(float(v)) for v in row] for row in wl.bf16_bits_to_f32(Xb)]
    Wf = [[Fraction(float(v)) for v in row] for row in W]
    df = [Fraction(float(v)) for v in d]
    sgn = lambda i, j: -1 if bin(i & j).count("1") & 1 else 1
    Vun = [[sum(X[i][k] * df[k] * sgn(k, j) for k in range(K)) for j in range(K)] for i in range(M)]
    Wun = [[sum(sgn(k, j) * Wf[k][n] / df[k] for k in range(K)) for n in range(N)] for j in range(K)]
    Xq = [_brute_force_codes(Vun[i]) for i in range(M)]
    Wq_cols = [_brute_force_codes([Wun[k][n] for k in range(K)]) for n in range(N)]
    assert out["Xq"].tolist() == Xq
    assert out["Wq"].T.tolist() == Wq_cols
    acc = [[sum(Xq[i][k] * Wq_cols[n][k] for k in range(K)) for n in range(N)] for i in range(M)]
    assert out["acc"].tolist() == acc
    rb = 1 / np.sqrt(B)
    for i in range(M):
        sx = float(max(abs(v) for v in Vun[i])) * rb / 127
        assert out["sx"][i] == pytest.approx(sx, rel=1e-14)
        for n in range(N):
            sw = float(max(abs(Wun[k][n]) for k in range(K))) * rb / 127
            y = acc[i][n] * sx * sw + float(bias[n])
            assert out["Yd"][i, n] == pytest.approx(y, rel=1e-12, abs=1e-15)


def test_whole_path_w4_groups_brute_force(oracle):
    M, K, N, B = 3, 16, 5, 8                   # two groups of 8 input channels
    Xb, W, d, bias = wl.small_case(11, M, K, N, n_outliers=1, outlier=20.0)
    out = oracle.linear(Xb, W, d, bias, B=B, wbits=4)
    Wp = oracle.rotate_weights(W, d, B)
    assert out["sw"].shape == (2, N) and out["acc"].shape == (2, M, N)
    for g in range(2):
        for n in range(N):
            col = [Fraction(float(v)) for v in Wp[g * B:(g + 1) * B, n]]
            a = max(abs(v) for v in col)
            want = [_round_half_even_fraction(v * 7 / a) for v in col]
            assert out["Wq"][g * B:(g + 1) * B, n].tolist() == want
    Xq, Wq = out["Xq"].astype(int), out["Wq"].astype(int)
    for g in range(2):
        assert np.array_equal(out["acc"][g], Xq[:, g * B:(g + 1) * B] @ Wq[g * B:(g + 1) * B])
    y = out["sx"][:, None] * sum(out["sw"][g][None, :] * out["acc"][g] for g in range(2)) + bias
    assert np.allclose(out["Yd"], y, rtol=1e-14)


def test_single_c_entry_point_agrees_with_steps(oracle):
    Xb, W, d, bias = wl.small_case(2, 20, 256, 24)
    for wbits in (8, 4):
        a = oracle.linear(Xb, W, d, bias, wbits=wbits)["Y"]
        assert np.array_equal(a, oracle.linear_c(Xb, W, d, bias, wbits=wbits))


# --------------------------------------------------- end-to-end error behaviour

def test_quantised_output_close_to_exact_and_rotation_helps(oracle):
    """W8A8 on config-0 data: about 1% relative error, inside the analytic bound,
    and clearly better than the same quantiser without rotation (the paper's claim)."""
    cfg = wl.CONFIGS[0]
    Xb = wl.make_x(cfg, "proj", M=256)
    W = wl.make_w(cfg, "proj")[:, :256].copy()
    exact = wl.bf16_bits_to_f32(Xb).astype(np.float64) @ W.astype(np.float64)
    out = oracle.linear(Xb, W, None, None, wbits=8, exact_blas=True)
    rel = np.linalg.norm(out["Yd"] - exact) / np.linalg.norm(exact)
    assert rel < 0.02
    V, Wp = oracle.rotate(Xb), oracle.rotate_weights(W)
    sx, sw = out["sx"], out["sw"]
    bound = (0.5 * sx[:, None] * np.abs(Wp).sum(axis=0)[None, :]
             + 0.5 * sw[None, :] * np.abs(V).sum(axis=1)[:, None]
             + 0.25 * V.shape[1] * sx[:, None] * sw[None, :])
    assert np.all(np.abs(out["Yd"] - exact) <= bound * (1 + 1e-9))
    # no rotation: quantise X and W directly with the same quantisers
    Xf = wl.bf16_bits_to_f32(Xb).astype(np.float64)
    Xq0, sx0 = oracle.quant_tokens(Xf)
    Wq0, sw0 = oracle.quant_weights(W.astype(np.float64), 8, 128)
    _, Y0 = oracle.dequant(oracle.acc_exact_blas(Xq0, Wq0), sx0, sw0, None, return_f64=True)
    rel0 = np.linalg.norm(Y0 - exact) / np.linalg.norm(exact)
    assert rel0 > 2.5 * rel


# -------------------------------------------------------------- group table

@pytest.mark.parametrize("n_steps,n_groups", [(20, 5), (50, 10), (10, 10), (7, 3), (1, 1)])
def test_table_default_partition(oracle, n_steps, n_groups):
    m = oracle.table_default(n_steps, n_groups)
    assert m[0] == 0 and m[-1] == n_groups - 1
    assert np.all(np.diff(m) >= 0) and np.all(np.diff(m) <= 1)       # monotone, contiguous
    sizes = np.bincount(m, minlength=n_groups)
    assert sizes.max() - sizes.min() <= 1
    assert [wl.draw_group(type("C", (), dict(n_steps=n_steps, n_groups=n_groups)), s)
            for s in range(n_steps)] == m.tolist()


def test_table_default_rejects_bad_arguments(oracle):
    with pytest.raises(RuntimeError):
        oracle.table_default(3, 5)


# ------------------------------------------------------------ frozen fixtures

@pytest.mark.parametrize("name", ["tiny_w8a8_4x8x8.txt", "tiny_w4a8_3x16x5.txt"])
def test_oracle_matches_frozen_fixture(oracle, name):
    import importlib.util
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "make_golden.py"))
    mg = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mg)
    out = mg.compute(mg.CASES[name])
    rows = dict(line.split(" ", 1) for line in open(os.path.join(here, name)) if not line.startswith("#"))
    for key in ("Xq", "Wq", "acc"):
        assert out[key].reshape(-1).tolist() == [int(t) for t in rows[key].split()]
    assert [f"{v:04x}" for v in out["Y"].reshape(-1).tolist()] == rows["Y"].split()


# ------------------------------------- zigzag permutation and second rotation (Eq. 9)

def _read_fixture(name):
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    out = {}
    for line in open(os.path.join(here, name)):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        out[key] = [float(v) for v in vals]
    return out


def test_zigzag_hand_worked_example(oracle):
    fx = _read_fixture("zigzag_8ch_2blocks.txt")
    perm = oracle.zigzag(np.array(fx["mag"]), B=4)
    assert perm.tolist() == [int(v) for v in fx["perm"]]


def test_zigzag_is_a_balanced_permutation(oracle):
    rng = np.random.default_rng(5)
    K, B = 1152, 128
    mag = np.abs(rng.standard_normal(K))
    hot = rng.choice(K, size=8, replace=False)
    mag[hot] *= 50.0                                   # massive-outlier channels
    perm = oracle.zigzag(mag, B)
    assert sorted(perm.tolist()) == list(range(K))     # a permutation: P is orthogonal
    blocks = mag[perm].reshape(K // B, B)
    # every round deals one channel to every block, largest first: slot r of any block holds a
    # channel no smaller than slot r+1 of any block
    assert np.all(blocks[:, :-1].min(axis=0) >= blocks[:, 1:].max(axis=0))
    # the outliers are spread: no block gets two of the 8 before every block has one (9 blocks)
    assert np.all((blocks > 10 * np.median(mag)).sum(axis=1) <= 1)
    # two consecutive rounds give block i the ranks i and 2nb-1-i: block sums of sorted data
    # differ by at most the first round's spread
    sums = blocks.sum(axis=1)
    srt = np.sort(mag)[::-1]
    assert sums.max() - sums.min() <= srt[0] - srt[K // B - 1] + 1e-12
    # contiguous blocks of the same data are far less balanced
    contiguous = mag.reshape(K // B, B).sum(axis=1)
    assert sums.max() - sums.min() < contiguous.max() - contiguous.min()


def test_rpr_identity_permutation_undoes_the_rotation(oracle):
    # H_B is symmetric, so R R = I: with P = I, G_t(X) = X diag(d) exactly (up to rounding)
    rng = np.random.default_rng(6)
    M, K, B = 5, 256, 128
    X = _bf16(rng.standard_normal((M, K)))
    d = np.exp(0.3 * rng.standard_normal(K)).astype(np.float32)
    V = oracle.rotate_rpr(X, d, np.arange(K, dtype=np.int32), B)
    U = oracle.bf16_to_f64(X) * d.astype(np.float64)
    assert np.allclose(V, U, rtol=0, atol=1e-12 * np.abs(U).max())


def test_rpr_matches_dense_matrices(oracle):
    # G_t(X) = X D R P R with R and P written out as dense K x K matrices (library products)
    rng = np.random.default_rng(7)
    M, K, B = 6, 256, 128
    X = _bf16(rng.standard_normal((M, K)))
    d = np.exp(0.3 * rng.standard_normal(K)).astype(np.float32)
    perm = rng.permutation(K).astype(np.int32)
    Rb = scipy.linalg.hadamard(B) / np.sqrt(B)
    R = scipy.linalg.block_diag(*([Rb] * (K // B)))
    P = np.zeros((K, K))
    P[perm, np.arange(K)] = 1.0                        # (U P)[k'] = U[perm[k']]
    U = oracle.bf16_to_f64(X) * d.astype(np.float64)
    expect = U @ R @ P @ R
    V = oracle.rotate_rpr(X, d, perm, B)
    assert np.allclose(V, expect, rtol=0, atol=1e-12 * np.abs(expect).max())
    # norm preservation: R, P orthogonal
    assert np.allclose(np.linalg.norm(V, axis=1), np.linalg.norm(U, axis=1), rtol=1e-12)
    W = (0.02 * rng.standard_normal((K, 24))).astype(np.float32)
    Wp = oracle.rotate_weights_rpr(W, d, perm, B)
    expect_w = R.T @ P.T @ R.T @ (W.astype(np.float64) / d.astype(np.float64)[:, None])
    assert np.allclose(Wp, expect_w, rtol=0, atol=1e-12 * np.abs(expect_w).max())


def test_rpr_computational_invariance(oracle):
    # Eq. 9: [(X D) R P R] [R^T P^T R^T (D^-1 W)] = X W, unquantised, to 1e-9
    rng = np.random.default_rng(8)
    M, K, N, B = 16, 1152, 40, 128
    Xf = rng.standard_normal((M, K)).astype(np.float32)
    Xf[:, rng.choice(K, size=8, replace=False)] *= 50.0
    X = _bf16(Xf)
    d = np.exp(0.3 * rng.standard_normal(K)).astype(np.float32)
    W = (0.02 * rng.standard_normal((K, N))).astype(np.float32)
    V1 = oracle.rotate(X, d, B)
    perm = oracle.zigzag(np.abs(V1).max(axis=0), B)
    V = oracle.rotate_rpr(X, d, perm, B)
    Wp = oracle.rotate_weights_rpr(W, d, perm, B)
    exact = oracle.bf16_to_f64(X) @ W.astype(np.float64)
    assert np.abs(V @ Wp - exact).max() <= 1e-9 * np.abs(exact).max()


def test_rpr_balances_the_blocks(oracle):
    # what the permutation is for (Sec. 3.2): one block rotation leaves each block with its own
    # outliers' energy, so blocks differ widely; after the zigzag permutation and the second
    # rotation every block carries about the same energy
    rng = np.random.default_rng(9)
    M, K, B = 64, 1152, 128
    Xf = rng.standard_normal((M, K)).astype(np.float32)
    Xf[:, rng.choice(K, size=8, replace=False)] *= 50.0
    X = _bf16(Xf)
    V1 = oracle.rotate(X, None, B)
    perm = oracle.zigzag(np.abs(V1).max(axis=0), B)
    V2 = oracle.rotate_rpr(X, None, perm, B)
    e1 = (V1 ** 2).reshape(M, K // B, B).sum(axis=(0, 2))
    e2 = (V2 ** 2).reshape(M, K // B, B).sum(axis=(0, 2))
    assert np.isclose(e1.sum(), e2.sum(), rtol=1e-12)          # orthogonal: total energy kept
    assert e1.max() / e1.min() > 10.0                          # 8 outlier channels in 9 blocks
    assert e2.max() / e2.min() < 1.5


# ------------------------------------------------ calibration side (Eq. 5)

def test_smooth_diag_closed_forms(oracle):
    rng = np.random.default_rng(11)
    K = 64
    xmax = np.exp(rng.standard_normal(K) * 2.0)
    wmax = np.exp(rng.standard_normal(K))
    # alpha = 1: all of the range moves to the weights, every scaled activation channel peaks at 1
    d1 = oracle.smooth_diag(xmax, wmax, 1.0)
    assert np.allclose(xmax * d1, 1.0, rtol=1e-14)
    # alpha = 0: the other way round, every scaled weight row peaks at 1
    d0 = oracle.smooth_diag(xmax, wmax, 0.0)
    assert np.allclose(wmax / d0, 1.0, rtol=1e-14)
    # alpha = 1/2: both sides meet at the geometric mean
    dh = oracle.smooth_diag(xmax, wmax, 0.5)
    assert np.allclose(xmax * dh, np.sqrt(xmax * wmax), rtol=1e-14)
    assert np.allclose(wmax / dh, np.sqrt(xmax * wmax), rtol=1e-14)
    # Eq. 5 itself (Delta = 1 / d) for a general alpha
    a = 0.3
    assert np.allclose(1.0 / oracle.smooth_diag(xmax, wmax, a), xmax ** a / wmax ** (1 - a), rtol=1e-14)
    # dead channels keep d = 1
    xmax[3] = 0.0
    wmax[5] = 0.0
    d = oracle.smooth_diag(xmax, wmax, 0.5)
    assert d[3] == 1.0 and d[5] == 1.0 and np.all(np.isfinite(d))


def test_channel_statistics_on_data(oracle):
    rng = np.random.default_rng(12)
    M, K, N = 40, 256, 24
    Xf = rng.standard_normal((M, K)).astype(np.float32)
    Xf[:, 7] *= 60.0
    X = _bf16(Xf)
    W = (0.02 * rng.standard_normal((K, N))).astype(np.float32)
    xmax = oracle.channel_absmax(X)
    assert np.array_equal(xmax, np.abs(oracle.bf16_to_f64(X)).max(axis=0))
    assert xmax.argmax() == 7
    wmax = oracle.weight_row_absmax(W)
    assert np.array_equal(wmax, np.abs(W.astype(np.float64)).max(axis=1))
    # with d from Eq. 5 at alpha = 1/2 the scaled operands have equal per-channel maxima, and
    # the product is unchanged (Eq. 4)
    d = oracle.smooth_diag(xmax, wmax, 0.5)
    assert np.allclose(oracle.channel_absmax(X, d), oracle.weight_row_absmax(W / d[:, None]), rtol=1e-6)
    Xs = oracle.bf16_to_f64(X) * d
    assert np.allclose(Xs @ (W / d[:, None]), oracle.bf16_to_f64(X) @ W.astype(np.float64), rtol=1e-9, atol=1e-12)
    # rotated statistic: the maximum over tokens of the once-rotated activations
    mag = oracle.channel_absmax(X, d.astype(np.float32), rotate_first=True)
    assert np.array_equal(mag, np.abs(oracle.rotate(X, d.astype(np.float32), 128)).max(axis=0))


# ------------------------------------ asymmetric activation quantiser (Eq. 1-3)

def test_asym_quantiser_brute_force_rational(oracle):
    # Eq. 1-3 evaluated in exact rational arithmetic on a tiny input (values are dyadic, so the
    # float64 oracle must agree code for code)
    vals = [[-3.0, 1.5, 0.25, 2.0], [0.5, 4.0, 1.0, 0.125], [-1.0, -0.5, -4.0, -2.5], [0.0, 0.0, 0.0, 0.0]]
    V = np.array(vals, dtype=np.float64)
    Xq, sx, zx = oracle.quant_tokens_asym(V)

    def rne(fr):
        fl = fr.numerator // fr.denominator
        rem = fr - fl
        if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
            return fl + 1
        return fl
    for i, row in enumerate(vals):
        fr = [Fraction(v) for v in row]
        lo, hi = min(min(fr), Fraction(0)), max(max(fr), Fraction(0))
        if hi == lo:
            assert sx[i] == 0 and zx[i] == 0 and not Xq[i].any()
            continue
        s = (hi - lo) / 255
        z = -rne(lo / s)
        assert zx[i] == z and 0 <= z <= 255
        assert sx[i] == float(s)
        for k, v in enumerate(fr):
            assert Xq[i, k] == min(255, max(0, rne(v / s) + z))


def test_asym_quantiser_properties(oracle):
    rng = np.random.default_rng(21)
    M, K = 64, 256
    V = rng.standard_normal((M, K)) * np.exp(rng.standard_normal((M, 1)))
    V[3] = np.abs(V[3])                 # a non-negative row: lo = 0, z = 0
    V[4] = -np.abs(V[4])                # a non-positive row: hi = 0, z = 255
    V[5] = 7.0                          # a constant row: range [0, 7]
    Xq, sx, zx = oracle.quant_tokens_asym(V)
    assert zx[3] == 0 and zx[4] == 255 and zx[5] == 0 and np.all(Xq[5] == 255)
    # rows that straddle zero use the whole range; one-sided rows reach the end they have
    two_sided = np.ones(M, dtype=bool)
    two_sided[[3, 4, 5]] = False
    assert np.all(Xq[two_sided].min(axis=1) == 0) and np.all(Xq[two_sided].max(axis=1) == 255)
    assert Xq[3].max() == 255 and Xq[4].min() == 0
    deq = sx[:, None] * (Xq.astype(np.float64) - zx[:, None])
    assert np.all(np.abs(deq - V) <= 0.5 * sx[:, None] * (1 + 1e-9) + 0.5 * sx[:, None])   # rounding + zero-point rounding
    # twice the resolution of the symmetric quantiser on a one-sided row
    Xs, ss = oracle.quant_tokens(V[3:4])
    assert sx[3] < 0.51 * ss[0]
    # re-quantising the dequantised values reproduces the codes
    Xq2, sx2, zx2 = oracle.quant_tokens_asym(deq)
    assert np.array_equal(Xq2, Xq) and np.array_equal(zx2, zx)


def test_asym_integer_product_is_the_product_of_dequantised_operands(oracle):
    rng = np.random.default_rng(22)
    M, K, N = 5, 64, 7
    Xq = rng.integers(0, 256, size=(M, K)).astype(np.uint8)
    zx = rng.integers(0, 256, size=M).astype(np.int32)
    Wq = rng.integers(-127, 128, size=(K, N)).astype(np.int8)
    acc = oracle.igemm_asym(Xq, zx, Wq)
    brute = np.zeros((M, N), dtype=np.int64)
    for i in range(M):
        for n in range(N):
            brute[i, n] = sum((int(Xq[i, k]) - int(zx[i])) * int(Wq[k, n]) for k in range(K))
    assert np.array_equal(acc.astype(np.int64), brute)
    assert np.array_equal(oracle.acc_asym_exact_blas(Xq, zx, Wq), acc)
    # the form an int8 matrix unit can evaluate: signed codes q - 128 plus a column-sum correction
    colsum = Wq.astype(np.int64).sum(axis=0)
    signed = (Xq.astype(np.int64) - 128) @ Wq.astype(np.int64) + (128 - zx.astype(np.int64))[:, None] * colsum[None, :]
    assert np.array_equal(signed, brute)


def test_asym_linear_close_to_exact_product(oracle):
    rng = np.random.default_rng(23)
    M, K, N = 32, 1152, 48
    Xf = rng.standard_normal((M, K)).astype(np.float32)
    Xf[:, rng.choice(K, size=8, replace=False)] *= 50.0
    X = _bf16(Xf)
    W = (0.02 * rng.standard_normal((K, N))).astype(np.float32)
    ref = oracle.linear_asym(X, W)
    exact = oracle.bf16_to_f64(X) @ W.astype(np.float64)
    rel_a = np.linalg.norm(ref["Yd"] - exact) / np.linalg.norm(exact)
    rel_s = np.linalg.norm(oracle.linear(X, W)["Yd"] - exact) / np.linalg.norm(exact)
    assert rel_a < 0.02 and rel_a < 1.2 * rel_s


# ------------------------------------ asymmetric weight quantiser (Eq. 1-3 on H_t(W), per output channel)

@pytest.mark.parametrize("bits", [4, 6, 8])
def test_asym_weight_quantiser_brute_force_rational(oracle, bits):
    # exact rational arithmetic on dyadic values: the float64 oracle must agree code for code
    cols = [[-3.0, 1.5, 0.25, 2.0, -0.75], [0.5, 4.0, 1.0, 0.125, 2.5], [-1.0, -0.5, -4.0, -2.5, -0.25],
            [0.0, 0.0, 0.0, 0.0, 0.0]]
    Wp = np.array(cols, dtype=np.float64).T.copy()           # [K = 5, N = 4]: one list per output channel
    Wq, sw, zw = oracle.quant_weights_asym(Wp, bits)
    qmax = 2 ** bits - 1

    def rne(fr):
        fl = fr.numerator // fr.denominator
        rem = fr - fl
        return fl + 1 if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1) else fl
    for n, col in enumerate(cols):
        fr = [Fraction(v) for v in col]
        lo, hi = min(min(fr), Fraction(0)), max(max(fr), Fraction(0))
        if hi == lo:
            assert sw[n] == 0 and zw[n] == 0 and not Wq[:, n].any()
            continue
        s = (hi - lo) / qmax
        z = -rne(lo / s)
        assert zw[n] == z and 0 <= z <= qmax and sw[n] == float(s)
        for k, v in enumerate(fr):
            assert Wq[k, n] == min(qmax, max(0, rne(v / s) + z))


def test_asym_weight_quantiser_properties(oracle):
    rng = np.random.default_rng(31)
    K, N = 256, 48
    Wp = rng.standard_normal((K, N)) * 0.02 + rng.normal(0, 0.02, (1, N))     # columns with a non-zero mean
    Wp[:, 3] = np.abs(Wp[:, 3])             # one-sided columns
    Wp[:, 4] = -np.abs(Wp[:, 4])
    Wp[:, 5] = 0.0
    Wq, sw, zw = oracle.quant_weights_asym(Wp, 8)
    assert zw[3] == 0 and zw[4] == 255 and zw[5] == 0 and sw[5] == 0 and not Wq[:, 5].any()
    live = np.ones(N, dtype=bool); live[[3, 4, 5]] = False
    both = live & (Wp.min(axis=0) < 0) & (Wp.max(axis=0) > 0)       # columns that straddle zero use the whole range
    assert both.sum() > N // 2
    assert np.all(Wq[:, both].min(axis=0) == 0) and np.all(Wq[:, both].max(axis=0) == 255)
    deq = sw[None, :] * (Wq.astype(np.float64) - zw[None, :])
    assert np.all(np.abs(deq - Wp) <= sw[None, :] * (1 + 1e-9))             # rounding + zero-point rounding
    # a column with a large mean is resolved finer than by the symmetric quantiser (range hi - lo < 2 absmax)
    Ws, ss = oracle.quant_weights(Wp, 8)
    assert np.all(sw[live] * 255 <= ss[live] * 254 * (1 + 1e-12))
    assert np.mean((deq[:, live] - Wp[:, live]) ** 2) < np.mean((ss[live] * Ws[:, live] - Wp[:, live]) ** 2)
    # re-quantising the dequantised values reproduces the codes
    Wq2, sw2, zw2 = oracle.quant_weights_asym(deq, 8)
    assert np.array_equal(Wq2, Wq) and np.array_equal(zw2, zw)


def test_asym2_integer_product_is_the_product_of_dequantised_operands(oracle):
    rng = np.random.default_rng(32)
    M, K, N = 5, 64, 7
    Wq = rng.integers(0, 256, size=(K, N)).astype(np.uint8)
    zw = rng.integers(0, 256, size=N).astype(np.int32)
    for act_asym in (False, True):
        if act_asym:
            Xq = rng.integers(0, 256, size=(M, K)).astype(np.int16)
            zx = rng.integers(0, 256, size=M).astype(np.int32)
        else:
            Xq = rng.integers(-127, 128, size=(M, K)).astype(np.int16)
            zx = None
        acc = oracle.igemm_asym2(Xq, zx, Wq, zw)
        zi = np.zeros(M, dtype=np.int64) if zx is None else zx.astype(np.int64)
        brute = np.zeros((M, N), dtype=np.int64)
        for i in range(M):
            for n in range(N):
                brute[i, n] = sum((int(Xq[i, k]) - int(zi[i])) * (int(Wq[k, n]) - int(zw[n])) for k in range(K))
        assert np.array_equal(acc.astype(np.int64), brute)
        assert np.array_equal(oracle.acc_asym2_exact_blas(Xq, zx, Wq, zw), acc)
        # the form an int8 matrix unit evaluates: signed codes (q - 128) on both sides (activations as they are
        # when symmetric) plus the rank-one corrections with the row sums and column sums of the signed codes
        xs = Xq.astype(np.int64) - (128 if act_asym else 0)
        zcx = (128 - zi) if act_asym else np.zeros(M, dtype=np.int64)
        ws = Wq.astype(np.int64) - 128
        zcw = 128 - zw.astype(np.int64)
        signed = (xs @ ws + zcx[:, None] * ws.sum(axis=0)[None, :] + xs.sum(axis=1)[:, None] * zcw[None, :]
                  + K * zcx[:, None] * zcw[None, :])
        assert np.array_equal(signed, brute)
    # symmetric weights are the special case z = 128 of the signed form: reduces to the pinned igemm_asym
    Xq = rng.integers(0, 256, size=(M, K)).astype(np.uint8)
    zx = rng.integers(0, 256, size=M).astype(np.int32)
    Ws = rng.integers(-127, 128, size=(K, N)).astype(np.int8)
    assert np.array_equal(oracle.igemm_asym2(Xq.astype(np.int16), zx, (Ws.astype(np.int16) + 128).astype(np.uint8),
                                             np.full(N, 128, np.int32)), oracle.igemm_asym(Xq, zx, Ws))


@pytest.mark.parametrize("act_asym", [False, True])
def test_asym_weights_linear_close_to_exact_product(oracle, act_asym):
    rng = np.random.default_rng(33)
    M, K, N = 32, 1152, 48
    Xf = rng.standard_normal((M, K)).astype(np.float32)
    Xf[:, rng.choice(K, size=8, replace=False)] *= 50.0
    X = _bf16(Xf)
    W = (0.02 * rng.standard_normal((K, N))).astype(np.float32)
    ref = oracle.linear_asym_weights(X, W, act_asym=act_asym)
    exact = oracle.bf16_to_f64(X) @ W.astype(np.float64)
    rel_a = np.linalg.norm(ref["Yd"] - exact) / np.linalg.norm(exact)
    rel_s = np.linalg.norm(oracle.linear(X, W)["Yd"] - exact) / np.linalg.norm(exact)
    assert rel_a < 0.02 and rel_a < 1.2 * rel_s
    # the plain loop and the exact library product agree bit for bit
    ref2 = oracle.linear_asym_weights(X, W, act_asym=act_asym, exact_blas=True)
    assert np.array_equal(ref["acc"], ref2["acc"]) and np.array_equal(ref["Y"], ref2["Y"])


def test_rpr_asym_reduces_to_its_parts(oracle):
    # with the identity permutation the two Hadamard rotations cancel (H is symmetric and orthogonal), so the
    # Eq. 9 transform is X . Delta and its asymmetric codes are those of the plain quantiser on X . Delta;
    # with a real permutation the product stays close to the exact one
    rng = np.random.default_rng(41)
    M, K, N = 24, 256, 32
    Xf = rng.standard_normal((M, K)).astype(np.float32)
    Xf[:, 5] *= 30.0
    X = _bf16(Xf)
    d = rng.lognormal(0, 0.3, K).astype(np.float32)
    W = (0.02 * rng.standard_normal((K, N))).astype(np.float32)
    ident = np.arange(K, dtype=np.int32)
    ref = oracle.linear_rpr_asym(X, W, d, ident)
    V = oracle.bf16_to_f64(X) * d.astype(np.float64)[None, :]
    Xq, sx, zx = oracle.quant_tokens_asym(V)
    assert np.array_equal(ref["zx"], zx) and np.mean(ref["Xq"] != Xq) < 1e-3 and np.allclose(ref["sx"], sx, rtol=1e-12)
    perm = oracle.zigzag(np.abs(oracle.rotate(X, d, 128)).max(axis=0), 128).astype(np.int32)
    ref = oracle.linear_rpr_asym(X, W, d, perm)
    exact = oracle.bf16_to_f64(X) @ W.astype(np.float64)
    assert np.linalg.norm(ref["Yd"] - exact) / np.linalg.norm(exact) < 0.02
    assert np.array_equal(ref["acc"], oracle.linear_rpr_asym(X, W, d, perm, exact_blas=True)["acc"])


# ------------------------------------ other bit-widths (the W6A6 of Table 3)

@pytest.mark.parametrize("bits", [2, 4, 6, 7, 8])
def test_quant_tokens_bits_brute_force_rational(oracle, bits):
    # Eq. 1-2 (symmetric) in exact rational arithmetic on dyadic values, ties included
    qmax = 2 ** (bits - 1) - 1
    vals = [[-3.0, 1.5, 0.25, 2.0, 0.75], [0.5, 4.0, 1.0, 0.125, -4.0], [float(qmax), 0.5, 1.5, -2.5, -0.5],
            [0.0, 0.0, 0.0, 0.0, 0.0]]
    Xq, sx = oracle.quant_tokens_bits(np.array(vals), bits)

    def rne(fr):
        fl = fr.numerator // fr.denominator
        rem = fr - fl
        return fl + 1 if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1) else fl
    for i, row in enumerate(vals):
        fr = [Fraction(v) for v in row]
        a = max(abs(v) for v in fr)
        if a == 0:
            assert sx[i] == 0 and not Xq[i].any()
            continue
        s = a / qmax
        assert sx[i] == float(s)
        for k, v in enumerate(fr):
            assert Xq[i, k] == min(qmax, max(-qmax, rne(v / s)))
    if qmax >= 3:                                           # scale exactly 1: the halves go to the even neighbour
        assert sx[2] == 1.0 and Xq[2].tolist() == [qmax, 0, 2, -2, 0]


def test_quant_tokens_bits_reduces_to_the_8_bit_quantiser(oracle):
    V = oracle.rotate(wl.make_x(wl.CONFIGS[0], "proj", M=64))
    V[7] = 0.0
    a, sa = oracle.quant_tokens(V)
    b, sb = oracle.quant_tokens_bits(V, 8)
    assert np.array_equal(a, b) and np.array_equal(sa, sb)


def test_six_bit_quantisers_properties(oracle):
    B, K, N = 128, 256, 24
    Xb, W, d, _ = wl.small_case(17, 32, K, N)
    V = oracle.rotate(Xb, d, B)
    Xq, sx = oracle.quant_tokens(V, abits=6)
    assert np.all(np.abs(Xq).max(axis=1) == 31) and np.all(np.abs(Xq) <= 31)
    assert np.allclose(sx, np.abs(V).max(axis=1) / 31, rtol=1e-15)
    assert np.all(np.abs(V - sx[:, None] * Xq) <= sx[:, None] * (0.5 + 1e-12))
    Wp = oracle.rotate_weights(W, d, B)
    Wq, sw = oracle.quant_weights(Wp, 6, B)
    assert sw.shape == (N,) and np.all(np.abs(Wq).max(axis=0) == 31)
    assert np.allclose(sw, np.abs(Wp).max(axis=0) / 31, rtol=1e-15)
    assert np.all(np.abs(Wp - sw * Wq) <= sw * (0.5 + 1e-12))
    # fewer levels, larger error: W6A6 sits between W8A8 and the exact product
    exact = oracle.bf16_to_f64(Xb) @ W.astype(np.float64)
    e8 = np.abs(oracle.linear(Xb, W, d)["Yd"] - exact).mean()
    e6 = np.abs(oracle.linear(Xb, W, d, wbits=6, abits=6)["Yd"] - exact).mean()
    assert e8 < e6 < 8 * e8


# ------------------------------------ attention sharing (Sec. 3.3, Eq. 11)

def test_cosine_similarity_closed_forms(oracle):
    f = wl.f32_to_bf16_bits
    a = np.array([[1.0, 0.0, 0.0, 0.0], [3.0, 4.0, 0.0, 0.0], [1.0, 2.0, -2.0, 0.5], [0.0, 0.0, 0.0, 0.0]], dtype=np.float32)
    b = np.array([[0.0, 1.0, 0.0, 0.0], [1.0, 0.0, 0.0, 0.0], [1.0, 2.0, -2.0, 0.5], [1.0, 2.0, 3.0, 4.0]], dtype=np.float32)
    c = oracle.cosine_similarity(f(a), f(b))
    assert c[0] == 0.0                       # orthogonal
    assert abs(c[1] - 0.6) < 1e-15           # the 3-4-5 triangle
    assert abs(c[2] - 1.0) < 1e-15           # identical
    assert c[3] == 0.0                       # a zero vector has no direction
    assert abs(oracle.cosine_similarity(f(a[2:3]), f(-b[2:3]))[0] + 1.0) < 1e-15
    # scale invariance (powers of two keep bf16 values exact) and symmetry
    rng = np.random.default_rng(5)
    x = f(rng.standard_normal((3, 257)).astype(np.float32))
    y = f(rng.standard_normal((3, 257)).astype(np.float32))
    c0 = oracle.cosine_similarity(x, y)
    xs = f((oracle.bf16_to_f64(x) * 4.0).astype(np.float32))
    ys = f((oracle.bf16_to_f64(y) * 0.125).astype(np.float32))
    assert np.allclose(oracle.cosine_similarity(xs, ys), c0, rtol=0, atol=1e-15)
    assert np.array_equal(oracle.cosine_similarity(y, x), c0)
    assert np.all(np.abs(c0) <= 1.0)


def test_cosine_similarity_exact_rational(oracle):
    # cos^2 is rational: dot^2 / (|A|^2 |B|^2) in exact arithmetic on dyadic values
    a = [[1.5, -2.0, 0.25, 3.0, 0.5], [0.75, 0.5, -1.0, 2.0, 4.0]]
    b = [[0.5, 1.0, -4.0, 2.0, 0.125], [3.0, -0.25, 1.0, 1.0, 2.0]]
    c = oracle.cosine_similarity(wl.f32_to_bf16_bits(np.array(a, dtype=np.float32)),
                                 wl.f32_to_bf16_bits(np.array(b, dtype=np.float32)))
    for i in range(2):
        fa, fb = [Fraction(v) for v in a[i]], [Fraction(v) for v in b[i]]
        dot = sum(x * y for x, y in zip(fa, fb))
        c2 = dot * dot / (sum(x * x for x in fa) * sum(y * y for y in fb))
        assert abs(c[i] * c[i] - float(c2)) < 1e-15 and (c[i] > 0) == (dot > 0)


def test_share_plan(oracle):
    sim = np.array([[0.99, 0.70, 0.95, 0.999],
                    [0.97, 0.99, 0.95, 0.98],
                    [0.96, 0.99, 0.94, 0.97]])
    assert oracle.share_plan(sim, 0.95).tolist() == [1, 0, 0, 1]
    assert oracle.share_plan(sim, 0.5).tolist() == [1, 1, 1, 1]
    assert oracle.share_plan(sim, 0.96).tolist() == [1, 0, 0, 1]
    assert oracle.share_plan(sim, 1.0).tolist() == [0, 0, 0, 0]


# ------------------------------------ greedy dense block rotations (Eq. 6-7)

def test_dense_rotation_with_hadamard_blocks_is_the_fast_path(oracle):
    Xb, W, d, _ = wl.small_case(23, 24, 256, 16)
    Hn = oracle.hadamard(128).astype(np.float64) / np.sqrt(128.0)
    Rs = np.stack([Hn, Hn])
    assert np.allclose(oracle.rotate_dense(Xb, d, Rs), oracle.rotate(Xb, d, 128), rtol=0, atol=1e-9)
    assert np.allclose(oracle.rotate_weights_dense(W, d, Rs), oracle.rotate_weights(W, d, 128), rtol=0, atol=1e-12)


def test_dense_rotation_computational_invariance(oracle):
    # non-symmetric orthogonal blocks: a transposed operand on either side breaks the identity
    Xb, W, d, _ = wl.small_case(24, 20, 384, 24)
    Rs = wl.orthogonal_uniform_first_row(1, 3)
    assert np.abs(Rs[0] - Rs[0].T).max() > 0.1
    V = oracle.rotate_dense(Xb, d, Rs)
    Wp = oracle.rotate_weights_dense(W, d, Rs)
    exact = oracle.bf16_to_f64(Xb) @ W.astype(np.float64)
    assert np.allclose(V @ Wp, exact, rtol=0, atol=1e-9)
    # block b of V only depends on block b of X
    X2 = oracle.bf16_to_f64(Xb).copy(); X2[:, 128:256] = 0
    V2 = oracle.rotate_dense(wl.f32_to_bf16_bits(X2.astype(np.float32)), d, Rs)
    assert np.array_equal(V2[:, :128], V[:, :128]) and not V2[:, 128:256].any()


def test_drawn_matrices_are_orthogonal_with_uniform_first_row():
    Qs = wl.orthogonal_uniform_first_row(2, 4, 128)
    for Q in Qs:
        assert np.allclose(Q @ Q.T, np.eye(128), atol=1e-12)
        assert np.allclose(Q[0], 1 / np.sqrt(128.0), atol=1e-12)


def test_greedy_rotation_single_outlier_closed_form(oracle):
    # one massive channel: C1 brings it to column 0, the uniform first row of Q spreads it evenly, so
    # after one step every entry of a row has magnitude a / sqrt(B) (and C2 only moves two columns)
    B, a = 128, 640.0
    X = np.zeros((5, B)); X[:, 37] = a * np.array([1.0, -0.5, 0.25, 1.0, -1.0])
    Qs = wl.orthogonal_uniform_first_row(3, 1, B)
    R, n, m = oracle.greedy_rotation(X, Qs)
    assert n == 1 and abs(m[0] - a / np.sqrt(B)) < 1e-9
    assert np.allclose(np.abs(X @ R), np.abs(X[:, 37:38]) / np.sqrt(B) * np.ones((1, B)), atol=1e-9)


def test_greedy_rotation_properties(oracle):
    B, N = 128, 12
    rng = np.random.default_rng(8)
    X = rng.standard_normal((96, B)); X[:, [5, 77]] *= 60.0; X[3, 100] = 900.0
    Qs = wl.orthogonal_uniform_first_row(4, N, B)
    R, n, m = oracle.greedy_rotation(X, Qs)
    assert np.allclose(R @ R.T, np.eye(B), atol=1e-10)              # a product of orthogonal matrices
    assert 1 <= n <= N and m[n - 1] == m.min() and np.all(m[:n - 1] > m[n - 1])   # first minimum (Eq. 7)
    assert abs(np.abs(X @ R).max() - m[n - 1]) < 1e-9
    assert m[n - 1] < 0.25 * np.abs(X).max()                        # the outliers are gone
    # Eq. 6 by hand for the first step: explicit switching matrices around Q_1
    j = int(np.argmax(np.abs(X).max(axis=0)))
    assert j == 100
    C = np.eye(B); C[0, 0] = C[j, j] = 0; C[0, j] = C[j, 0] = 1
    R1, n1, m1 = oracle.greedy_rotation(X, Qs[:1])
    assert n1 == 1 and np.allclose(R1, C @ Qs[0] @ C, atol=1e-13)
    # Frobenius norm (energy) is preserved
    assert abs(np.linalg.norm(X @ R) - np.linalg.norm(X)) < 1e-8


def test_greedy_rotation_small_block_brute_force(oracle):
    # B = 4, two steps, every product written out element by element
    B = 4
    X = np.array([[1.0, -8.0, 0.5, 2.0], [0.25, 4.0, -1.0, 0.5]])
    Qs = wl.orthogonal_uniform_first_row(5, 2, B)

    def matmul(A, Bm):
        out = [[0.0] * len(Bm[0]) for _ in A]
        for i in range(len(A)):
            for jj in range(len(Bm[0])):
                out[i][jj] = sum(A[i][k] * Bm[k][jj] for k in range(len(Bm)))
        return out

    def swap_cols(A, j):
        out = [row[:] for row in A]
        for row in out:
            row[0], row[j] = row[j], row[0]
        return out
    Xc, Rc, ms, Rs_ = X.tolist(), np.eye(B).tolist(), [], []
    for Q in Qs:
        col_max = [max(abs(row[j]) for row in Xc) for j in range(B)]
        j = col_max.index(max(col_max))
        Xc = swap_cols(matmul(swap_cols(Xc, j), Q.tolist()), j)      # X C1 Q C2
        Rc = swap_cols(matmul(swap_cols(Rc, j), Q.tolist()), j)
        ms.append(max(abs(v) for row in Xc for v in row)); Rs_.append(np.array(Rc))
    R, n, m = oracle.greedy_rotation(X, Qs)
    assert np.allclose(m, ms, atol=1e-14)
    assert n == ms.index(min(ms)) + 1 and np.allclose(R, Rs_[n - 1], atol=1e-14)


# ------------------------------------ Eq. 10 in full with dense blocks (R1, P, R2)

def test_dense_rpr_reduces_to_the_hadamard_form(oracle):
    Xb, W, d, _ = wl.small_case(25, 24, 384, 16)
    Hn = oracle.hadamard(128).astype(np.float64) / np.sqrt(128.0)
    Rs = np.stack([Hn] * 3)
    perm = oracle.zigzag(np.abs(oracle.rotate(Xb, d, 128)).max(axis=0), 128)
    assert np.allclose(oracle.rotate_dense_rpr(Xb, d, Rs, perm, Rs), oracle.rotate_rpr(Xb, d, perm, 128), rtol=0, atol=1e-9)
    assert np.allclose(oracle.rotate_weights_dense_rpr(W, d, Rs, perm, Rs), oracle.rotate_weights_rpr(W, d, perm, 128),
                       rtol=0, atol=1e-12)


def test_dense_rpr_computational_invariance(oracle):
    Xb, W, d, _ = wl.small_case(26, 20, 384, 24)
    R1, R2 = wl.orthogonal_uniform_first_row(6, 3), wl.orthogonal_uniform_first_row(7, 3)
    perm = np.random.default_rng(4).permutation(384).astype(np.int32)
    V = oracle.rotate_dense_rpr(Xb, d, R1, perm, R2)
    Wp = oracle.rotate_weights_dense_rpr(W, d, R1, perm, R2)
    exact = oracle.bf16_to_f64(Xb) @ W.astype(np.float64)
    assert np.allclose(V @ Wp, exact, rtol=0, atol=1e-9)
    # the three factors as explicit K x K matrices
    K = 384
    def blockdiag(Rs):
        M = np.zeros((K, K))
        for b in range(3):
            M[b * 128:(b + 1) * 128, b * 128:(b + 1) * 128] = Rs[b]
        return M
    P = np.zeros((K, K)); P[perm, np.arange(K)] = 1.0          # (U P)[k'] = U[perm[k']]
    G = np.diag(d.astype(np.float64)) @ blockdiag(R1) @ P @ blockdiag(R2)
    assert np.allclose(V, oracle.bf16_to_f64(Xb) @ G, rtol=0, atol=1e-9)
    Hm = blockdiag(R2).T @ P.T @ blockdiag(R1).T @ np.diag(1.0 / d.astype(np.float64))
    assert np.allclose(Wp, Hm @ W.astype(np.float64), rtol=0, atol=1e-12)


def test_time_rotation_calibration_flattens_outliers(oracle):
    Xb, _, d, _ = wl.small_case(27, 128, 256, 16, n_outliers=3, outlier=60.0)
    Q1, Q2 = wl.orthogonal_uniform_first_row(8, 10), wl.orthogonal_uniform_first_row(9, 10)
    R1, n1, perm, R2, n2 = oracle.calibrate_time_rotation(Xb, d, Q1, Q2)
    assert sorted(perm.tolist()) == list(range(256))
    for Rs in (R1, R2):
        for b in range(2):
            assert np.abs(Rs[b].astype(np.float64) @ Rs[b].astype(np.float64).T - np.eye(128)).max() < 1e-5
    raw = np.abs(oracle.bf16_to_f64(Xb) * d).max()
    one = np.abs(oracle.rotate_dense(Xb, d, R1)).max()
    two = np.abs(oracle.rotate_dense_rpr(Xb, d, R1, perm, R2)).max()
    assert one < 0.3 * raw and two < 0.3 * raw


def test_asym_int4_groups(oracle):
    # asymmetric activations against int4 weights: per-group sums of (q - z) w; the signed-code / column-sum
    # identity holds group by group, and the result is the float product of the dequantised operands
    Xb, W, d, bias = wl.small_case(28, 6, 256, 16, n_outliers=2)
    ref = oracle.linear_asym(Xb, W, d, bias, wbits=4)
    Xq, zx, Wq, sw, sx = ref["Xq"], ref["zx"], ref["Wq"], ref["sw"], ref["sx"]
    assert ref["acc"].shape == (2, 6, 16) and sw.shape == (2, 16) and np.abs(Wq).max() == 7
    signed = oracle.igemm((Xq.astype(np.int16) - 128).astype(np.int8), Wq, 128)          # [2, 6, 16]
    colsum = Wq.astype(np.int64).reshape(2, 128, 16).sum(axis=1)                         # [2, 16]
    want = signed + (128 - zx.astype(np.int64))[None, :, None] * colsum[:, None, :]
    assert np.array_equal(ref["acc"], want)
    assert np.array_equal(ref["acc"], oracle.igemm_asym_groups(Xq, zx, Wq, 128, exact_blas=True))
    Xhat = sx[:, None] * (Xq.astype(np.float64) - zx[:, None])
    What = np.repeat(sw, 128, axis=0) * Wq
    assert np.allclose(ref["Yd"], Xhat @ What + bias, rtol=1e-12, atol=1e-12)
    # brute force of one entry
    i, n = 3, 5
    t = sum(sw[k // 128, n] * float((int(Xq[i, k]) - int(zx[i])) * int(Wq[k, n])) for k in range(256))
    assert abs(ref["Yd"][i, n] - (sx[i] * t + bias[n])) < 1e-9
