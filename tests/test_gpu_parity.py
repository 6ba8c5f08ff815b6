"""GPU parity: every kernel of libtrdq against the CPU oracle, element by element, through the
C ABI, on seeded inputs that span several tiles and ragged tails."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2503_06564_amd import trdq, workloads as wl  # noqa: E402
from tests import gpu_util as gu  # noqa: E402


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the MI355X; run them with -m gpu on the GPU box")
    trdq.lib()
    yield
    trdq.qgemm_set_variant(-1)


# ------------------------------------------------------------ rotate_quant

RQ_SHAPES = [(1, 128), (5, 256), (37, 1152), (130, 4608), (64, 128 * 13), (33, 128 * 25),
             (19, 128 * 47), (7, 128 * 64), (1000, 1152)]


@pytest.mark.parametrize("M,K", RQ_SHAPES)
@pytest.mark.parametrize("with_diag", [False, True])
def test_rotate_quant_matches_oracle(oracle, M, K, with_diag):
    say(f"rotate_quant M={M} K={K} diag={with_diag}")
    Xb, _, d, _ = wl.small_case(3, M, K, 16, n_outliers=max(1, K // 144))
    d = d if with_diag else None
    Xq, sx = gu.gpu_rotate_quant(Xb, d)
    want_q, want_s = oracle.rotate_quant(Xb, d)
    gu.assert_codes_close(Xq.cpu().numpy(), want_q, "Xq")
    gu.assert_scales_close(sx.cpu().numpy(), want_s, "s_x")


def test_rotate_quant_strided_rows_zero_rows_and_empty(oracle):
    say("rotate_quant strided / zero rows / empty")
    M, K = 70, 1152
    Xb, _, d, _ = wl.small_case(4, M, K, 16)
    Xb[3] = 0
    Xb[69] = 0x8000                       # a row of negative zeros
    Xq, sx = gu.gpu_rotate_quant(Xb, d, ldx=K + 64)
    want_q, want_s = oracle.rotate_quant(Xb, d)
    gu.assert_codes_close(Xq.cpu().numpy(), want_q, "Xq")
    gu.assert_scales_close(sx.cpu().numpy(), want_s, "s_x")
    assert sx[3].item() == 0 and sx[69].item() == 0 and int(Xq[3].abs().max()) == 0
    # M == 0: valid no-op
    Xq0, sx0 = gu.gpu_rotate_quant(np.zeros((0, K), np.uint16), d)
    assert Xq0.shape == (0, K) and sx0.shape == (0,)


def test_rotate_quant_closed_forms():
    say("rotate_quant closed forms")
    K = 256
    X = np.zeros((K + 1, K), dtype=np.float32)
    X[np.arange(K), np.arange(K)] = 3.0           # unit vectors: every code of the block +-127
    X[K, :128] = 0.5                              # constant block: only coefficient 0 survives
    Xq, sx = gu.gpu_rotate_quant(wl.f32_to_bf16_bits(X), None)
    Xq = Xq.cpu().numpy().astype(int)
    for k in (0, 1, 77, 128, 255):
        b = k // 128
        blk = Xq[k, b * 128:(b + 1) * 128]
        signs = np.array([-1 if bin((k % 128) & j).count("1") & 1 else 1 for j in range(128)])
        assert np.array_equal(blk, 127 * signs)
        assert np.all(np.delete(Xq[k].reshape(2, 128), b, axis=0) == 0)
    assert Xq[K, 0] == 127 and np.all(Xq[K, 1:] == 0)
    assert np.allclose(sx.cpu().numpy()[:K], 3.0 / np.sqrt(128) / 127, rtol=1e-6)


# --------------------------------------------------------- prepare_weights

@pytest.mark.parametrize("K,N", [(128, 16), (256, 48), (1152, 1152), (4608, 80), (384, 208)])
@pytest.mark.parametrize("wbits", [8, 4])
def test_prepare_weights_matches_oracle(oracle, K, N, wbits):
    say(f"prepare_weights K={K} N={N} wbits={wbits}")
    _, W, d, _ = wl.small_case(5, 4, K, N)
    W[:, N // 2] = 0.0                               # a dead output channel
    w = trdq.prepare_weights(gu.f32_to_dev(W), gu.f32_to_dev(d), wbits=wbits)
    assert w.info() == (K, N, wbits)
    codes, scales = w.export()
    want_q, want_s = oracle.prepare_weights(W, d, 128, wbits)
    gu.assert_codes_close(codes, want_q, "Wq")
    gu.assert_scales_close(scales, want_s, "s_w")
    assert np.all(codes[:, N // 2] == 0) and np.all(scales[..., N // 2] == 0)
    assert np.abs(codes).max() == (127 if wbits == 8 else 7)
    if wbits == 4:
        assert np.array_equal(w.export_packed(), oracle.pack_int4(codes))
        assert w.nbytes() == K * N // 2 + (K // 128) * N * 4
    else:
        with pytest.raises(trdq.TrdqError) as e:
            w.export_packed()
        assert e.value.status == trdq.ERR_MISMATCH
    w.close()


def test_prepare_weights_without_diag(oracle):
    _, W, _, _ = wl.small_case(6, 4, 256, 32)
    w = trdq.prepare_weights(gu.f32_to_dev(W), None, wbits=8)
    codes, scales = w.export()
    want_q, want_s = oracle.prepare_weights(W, None, 128, 8)
    gu.assert_codes_close(codes, want_q, "Wq")
    gu.assert_scales_close(scales, want_s, "s_w")


# ------------------------------------------------------------------ qgemm

def _linear_case(oracle, seed, M, K, N, wbits, variant, with_bias=True, ldy=None):
    """Runs the unfused GPU path and checks every stage against the oracle."""
    Xb, W, d, bias = wl.small_case(seed, M, K, N, n_outliers=max(1, K // 144))
    bias = bias if with_bias else None
    trdq.qgemm_set_variant(variant)
    w = trdq.prepare_weights(gu.f32_to_dev(W), gu.f32_to_dev(d), wbits=wbits)
    Xq, sx = gu.gpu_rotate_quant(Xb, d)
    Y, acc = gu.gpu_qgemm(w, Xq, sx, bias, N, debug=True, ldy=ldy)
    # (ii) accumulators bit-exact given the GPU's own codes
    Xq_h, (Wq_h, sw_h) = Xq.cpu().numpy(), w.export()
    group = None if wbits == 8 else 128
    want_acc = oracle.acc_exact_blas(Xq_h, Wq_h, group) if M * K * N > 2e8 else oracle.igemm(Xq_h, Wq_h, group)
    assert np.array_equal(acc.cpu().numpy(), want_acc), "int32 accumulators differ"
    # epilogue on the same codes and scales
    y_same = oracle.dequant(want_acc, sx.cpu().numpy(), sw_h, bias)
    gu.assert_y_same_codes(gu.bf16_to_host(Y), y_same, "Y (same codes)")
    # (i) codes and scales, (iii) outputs against the oracle's own end-to-end quantised result
    ref = oracle.linear(Xb, W, d, bias, wbits=wbits, exact_blas=True)
    gu.assert_codes_close(Xq_h, ref["Xq"], "Xq")
    gu.assert_codes_close(Wq_h, ref["Wq"], "Wq")
    gu.assert_scales_close(sx.cpu().numpy(), ref["sx"], "s_x")
    gu.assert_scales_close(sw_h, ref["sw"], "s_w")
    worst = gu.assert_y_close(gu.bf16_to_host(Y), ref["Y"], "Y (oracle end to end)",
                              *gu.narrow_code_masks(8, wbits, Xq_h, ref["Xq"], Wq_h, ref["Wq"]))
    # without the debug output the result is the same
    Y2, _ = gu.gpu_qgemm(w, Xq, sx, bias, N, debug=False, ldy=ldy)
    assert torch.equal(Y2, Y)
    w.close()
    return worst


GEMM_SHAPES = [(1, 128, 16), (17, 256, 144), (128, 1152, 128), (257, 1152, 1152), (300, 4608, 272),
               (513, 384, 400)]


@pytest.mark.parametrize("M,K,N", GEMM_SHAPES)
@pytest.mark.parametrize("variant", list(range(trdq.qgemm_num_variants())))
def test_qgemm_w8_all_variants(oracle, M, K, N, variant):
    say(f"qgemm W8 M={M} K={K} N={N} variant={variant}")
    _linear_case(oracle, 7, M, K, N, 8, variant)


# full-tile shapes for the software-pipelined kernels (variants 11..15), including K shorter
# than the stage ring (one and two k-tiles) and the real layer widths
PIPE_SHAPES = [(256, 128, 256), (512, 256, 256), (256, 1152, 512), (768, 384, 768), (512, 4608, 256), (2048, 512, 2304),
               (1024, 1152, 1152), (384, 640, 288), (512, 256, 288), (256, 1024, 288), (384, 4608, 144)]


@pytest.mark.parametrize("M,K,N", PIPE_SHAPES)
@pytest.mark.parametrize("variant", list(range(11, trdq.qgemm_num_variants())))
def test_qgemm_w8_pipelined_full_tiles(oracle, M, K, N, variant):
    say(f"qgemm W8 pipelined M={M} K={K} N={N} variant={variant}")
    _linear_case(oracle, 13, M, K, N, 8, variant)


# ragged token counts with the built-in choice: whole panels on the fast kernels, the remaining rows on the
# kernel that takes any shape (two launches); tails shorter and longer than 128 rows, 144- and 128-wide tiles
@pytest.mark.parametrize("M,K,N", [(1100, 1152, 1152), (1025, 256, 288), (2180, 384, 400), (1407, 2304, 144),
                                   (4100, 512, 1152)])
def test_qgemm_w8_ragged_tokens_split(oracle, M, K, N):
    say(f"qgemm W8 ragged tokens M={M} K={K} N={N}")
    _linear_case(oracle, 15, M, K, N, 8, -1)


def _random_shapes(n, seed):
    r = np.random.default_rng(seed)
    shapes = []
    for _ in range(n):
        M = int(r.choice([r.integers(1, 64), r.integers(64, 1200), r.integers(1200, 5000)]))
        K = 128 * int(r.integers(1, 13))
        N = int(r.choice([16 * r.integers(1, 80), 144 * r.integers(1, 9), 128 * r.integers(1, 10)]))
        shapes.append((M, K, N))
    return shapes


# seeded random shapes through the built-in choice: whatever kernel, split or fallback the shape selects
@pytest.mark.parametrize("M,K,N", _random_shapes(16, 2024))
@pytest.mark.parametrize("wbits", [8, 4])
def test_linear_random_shapes_builtin_choice(oracle, M, K, N, wbits):
    say(f"random shape M={M} K={K} N={N} wbits={wbits}")
    _linear_case(oracle, 16, M, K, N, wbits, -1)


# more output tiles than compute units (workgroups of the persistent kernels walk several
# tiles), with two and three k-tiles, ragged and full edges, both tile orders
@pytest.mark.parametrize("M,K,N", [(4352, 256, 4400), (4096, 384, 4608), (2304, 1152, 1152)])
@pytest.mark.parametrize("variant", [16, 20, trdq.qgemm_num_variants() - 1])
def test_qgemm_w8_persistent_many_tiles(oracle, M, K, N, variant):
    say(f"qgemm W8 persistent M={M} K={K} N={N} variant={variant}")
    _linear_case(oracle, 17, M, K, N, 8, variant)


@pytest.mark.parametrize("M,K,N", GEMM_SHAPES)
@pytest.mark.parametrize("variant", [1, 5, 6, 7])
def test_qgemm_w4_all_variants(oracle, M, K, N, variant):
    say(f"qgemm W4 M={M} K={K} N={N} variant={variant}")
    _linear_case(oracle, 8, M, K, N, 4, variant)


@pytest.mark.parametrize("M,K,N", PIPE_SHAPES)
@pytest.mark.parametrize("variant", [6, 7])
def test_qgemm_w4_direct_to_lds_full_tiles(oracle, M, K, N, variant):
    say(f"qgemm W4 direct-to-LDS M={M} K={K} N={N} variant={variant}")
    _linear_case(oracle, 14, M, K, N, 4, variant)


@pytest.mark.parametrize("wbits", [8, 4])
def test_qgemm_no_bias_strided_output_and_empty(oracle, wbits):
    say(f"qgemm no bias / strided Y / empty, wbits={wbits}")
    _linear_case(oracle, 9, 70, 256, 48, wbits, -1, with_bias=False, ldy=64)
    _, W, d, _ = wl.small_case(9, 4, 256, 48)
    w = trdq.prepare_weights(gu.f32_to_dev(W), gu.f32_to_dev(d), wbits=wbits)
    Xq = torch.zeros((0, 256), dtype=torch.int8, device="cuda")
    sx = torch.zeros((0,), dtype=torch.float32, device="cuda")
    Y, _ = gu.gpu_qgemm(w, Xq, sx, None, 48, debug=False)
    assert Y.shape == (0, 48)


def test_qgemm_extreme_accumulators(oracle):
    """All codes +-127 over K = 4608: the largest accumulator magnitude the path can see."""
    say("qgemm extreme accumulators")
    M, K, N = 16, 4608, 16
    # a column that is sqrt(128) at the head of every block rotates to all ones: codes all +-127
    W = np.zeros((K, N), dtype=np.float32)
    W[::128, :] = np.float32(np.sqrt(128.0))
    W[:, 1::2] *= -1.0
    w = trdq.prepare_weights(gu.f32_to_dev(W), None, wbits=8)
    Wq, _ = w.export()
    assert np.all(np.abs(Wq) == 127)
    Xq = torch.full((M, K), 127, dtype=torch.int8, device="cuda")
    Xq[1::2] = -127
    sx = torch.ones((M,), dtype=torch.float32, device="cuda")
    Y, acc = gu.gpu_qgemm(w, Xq, sx, None, N, debug=True)
    want = oracle.igemm(Xq.cpu().numpy(), Wq)
    assert np.array_equal(acc.cpu().numpy(), want)
    assert np.abs(want).max() == 127 * 127 * K


# ------------------------------------------------------------------ fused

@pytest.mark.parametrize("M,K,N", [(1, 128, 16), (70, 1152, 272), (257, 1152, 1152), (130, 2304, 144),
                                   (100, 4608, 400), (65, 1536, 128), (33, 128 * 25, 48)])
@pytest.mark.parametrize("wbits", [8, 4])
def test_fused_matches_unfused_and_oracle(oracle, M, K, N, wbits):
    say(f"fused M={M} K={K} N={N} wbits={wbits}")
    Xb, W, d, bias = wl.small_case(10, M, K, N, n_outliers=max(1, K // 144))
    trdq.qgemm_set_variant(-1)
    w = trdq.prepare_weights(gu.f32_to_dev(W), gu.f32_to_dev(d), wbits=wbits)
    Xq, sx = gu.gpu_rotate_quant(Xb, d)
    Y_unfused, _ = gu.gpu_qgemm(w, Xq, sx, bias, N, debug=False)
    X = gu.bf16_to_dev(Xb)
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    trdq.linear_fused(X, gu.f32_to_dev(d), w, Y, bias=gu.f32_to_dev(bias))
    torch.cuda.synchronize()
    # The fused kernel rotates with vector-ALU butterflies, rotate_quant with the matrix cores:
    # the same fp32 accuracy but another rounding order, so a code may differ by one LSB on a
    # rare element (the tolerance of both against the oracle); everything else is identical.
    same = (Y == Y_unfused).float().mean().item()
    assert same >= 0.98, f"fused and unfused paths agree on only {same:.4f} of the outputs"
    gu.assert_y_close(gu.bf16_to_host(Y), gu.bf16_to_host(Y_unfused), "fused vs unfused")
    ref = oracle.linear(Xb, W, d, bias, wbits=wbits, exact_blas=True)
    gu.assert_y_close(gu.bf16_to_host(Y), ref["Y"], "Y fused")
    w.close()


@pytest.mark.parametrize("K", [128, 256, 384, 640, 896, 1152, 1408, 1536])
@pytest.mark.parametrize("M,N", [(40, 144), (512, 288), (19, 160)])
def test_fused_few_token_kernel(oracle, M, K, N):
    """The 16-token-panel kernel (int8 weights, K <= 1536): every count of blocks per lane row,
    144- and 128-channel tiles, ragged token and channel counts."""
    say(f"fused few tokens M={M} K={K} N={N}")
    Xb, W, d, bias = wl.small_case(31, M, K, N, n_outliers=max(1, K // 144), outlier=40.0)
    w = trdq.prepare_weights(gu.f32_to_dev(W), gu.f32_to_dev(d), wbits=8)
    Y = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    trdq.linear_fused(gu.bf16_to_dev(Xb), gu.f32_to_dev(d), w, Y, bias=gu.f32_to_dev(bias))
    torch.cuda.synchronize()
    ref = oracle.linear(Xb, W, d, bias, wbits=8, exact_blas=True)
    gu.assert_y_close(gu.bf16_to_host(Y), ref["Y"], "Y fused (few tokens)")
    # no diagonal: the kernel fills ones itself
    w1 = trdq.prepare_weights(gu.f32_to_dev(W), None, wbits=8)
    trdq.linear_fused(gu.bf16_to_dev(Xb), None, w1, Y)
    torch.cuda.synchronize()
    ref1 = oracle.linear(Xb, W, None, None, wbits=8, exact_blas=True)
    gu.assert_y_close(gu.bf16_to_host(Y), ref1["Y"], "Y fused (few tokens, no diagonal, no bias)")
    w.close(); w1.close()


def test_layer_chooses_fused_for_few_tokens(oracle):
    """fused=None: few tokens take the fused kernel (no workspace needed), many take the pair."""
    K, N = 256, 288
    table = trdq.Table(4, 1)
    layer = trdq.Layer(table, K, N, 8)
    Xb, W, d, bias = wl.small_case(13, 4096, K, N)
    layer.set_group(0, gu.f32_to_dev(d), gu.f32_to_dev(W))
    for M, needs_ws in ((64, False), (4096, True)):
        X = gu.bf16_to_dev(Xb[:M])
        Y = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
        if needs_ws:
            with pytest.raises(trdq.TrdqError) as e:
                layer.forward(1, X, Y, fused=None)
            assert e.value.status == trdq.ERR_NULL
            Xq_ws = torch.empty((M, K), dtype=torch.int8, device="cuda")
            sx_ws = torch.empty((M,), dtype=torch.float32, device="cuda")
            layer.forward(1, X, Y, bias=gu.f32_to_dev(bias), fused=None, Xq_ws=Xq_ws, sx_ws=sx_ws)
        else:
            layer.forward(1, X, Y, bias=gu.f32_to_dev(bias), fused=None)
        torch.cuda.synchronize()
        ref = oracle.linear(Xb[:M], W, d, bias, wbits=8)
        gu.assert_y_close(gu.bf16_to_host(Y), ref["Y"], f"layer, library's choice, M={M}")
    layer.close()


def test_fused_rejects_wide_k():
    _, W, _, _ = wl.small_case(1, 1, 128 * 49, 16)
    w = trdq.prepare_weights(gu.f32_to_dev(W), None, wbits=8)
    X = torch.zeros((4, 128 * 49), dtype=torch.bfloat16, device="cuda")
    Y = torch.zeros((4, 16), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(trdq.TrdqError) as e:
        trdq.linear_fused(X, None, w, Y)
    assert e.value.status == trdq.ERR_UNSUPPORTED


# ------------------------------------------------------------------ layer

@pytest.mark.parametrize("wbits,fused", [(8, False), (8, True), (4, False), (4, True)])
def test_layer_time_step_groups(oracle, wbits, fused):
    """20 steps -> 5 groups: each step must use its own group's diagonal and weights (Eq. 10)."""
    say(f"layer wbits={wbits} fused={fused}")
    M, K, N = 48, 256, 64
    table = trdq.Table(20, 5)
    layer = trdq.Layer(table, K, N, wbits)
    Xb, W, _, bias = wl.small_case(12, M, K, N)
    diags = [np.random.default_rng(100 + g).lognormal(0, 0.3, K).astype(np.float32) for g in range(5)]
    for g in (0, 2, 4):
        layer.set_group(g, gu.f32_to_dev(diags[g]), gu.f32_to_dev(W))
    X = gu.bf16_to_dev(Xb)
    Xq_ws = torch.empty((M, K), dtype=torch.int8, device="cuda")
    sx_ws = torch.empty((M,), dtype=torch.float32, device="cuda")
    want_map = oracle.table_default(20, 5)             # the oracle's step -> group map, not the product's
    assert [table.lookup(s) for s in range(20)] == [int(v) for v in want_map]
    for step in (0, 3, 9, 19):
        g = int(want_map[step])
        Y = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
        layer.forward(step, X, Y, bias=gu.f32_to_dev(bias), fused=fused, Xq_ws=Xq_ws, sx_ws=sx_ws)
        torch.cuda.synchronize()
        ref = oracle.linear(Xb, W, diags[g], bias, wbits=wbits)
        gu.assert_y_close(gu.bf16_to_host(Y), ref["Y"], f"layer step {step}")
        codes, _ = layer.weights(g).export()
        gu.assert_codes_close(codes, ref["Wq"], "layer Wq")
    with pytest.raises(trdq.TrdqError) as e:       # group 1 was never set
        layer.forward(5, X, Y, fused=fused, Xq_ws=Xq_ws, sx_ws=sx_ws)
    assert e.value.status == trdq.ERR_MISMATCH
    layer.close()


def test_graph_replay_matches_host_launches(oracle):
    """rotate_quant + qgemm captured into a HIP graph: every replay, with host-launched work and
    synchronisations between the replays, gives the bits of the host-launched path."""
    say("graph replay of rotate_quant + qgemm")
    M, K, N = 512, 1152, 1152
    trdq.qgemm_set_variant(-1)
    inputs = [wl.small_case(21 + i, M, K, N, n_outliers=8) for i in range(3)]
    Xb0, W, d, bias = inputs[0]
    w = trdq.prepare_weights(gu.f32_to_dev(W), gu.f32_to_dev(d), wbits=8)
    dd, bb = gu.f32_to_dev(d), gu.f32_to_dev(bias)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        X = gu.bf16_to_dev(Xb0).clone()
        Xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
        sx = torch.empty((M,), dtype=torch.float32, device="cuda")
        Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        rq = trdq.bind_rotate_quant(X, dd, Xq, sx, stream=s)
        mm = trdq.bind_qgemm(w, Xq, sx, Y, bias=bb, stream=s)
        rq(); mm()                      # warm-up outside the capture (one-time kernel attributes)
        s.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            rq(); mm()
        for Xb, _, _, _ in inputs:
            X.copy_(gu.bf16_to_dev(Xb))
            Y.zero_(); Xq.zero_()       # host-launched work between the replays
            g.replay()
            s.synchronize()
            got = (Xq.clone(), sx.clone(), Y.clone())
            Y.zero_(); Xq.zero_()
            rq(); mm()
            s.synchronize()
            assert torch.equal(got[0], Xq) and torch.equal(got[1], sx) and torch.equal(got[2], Y)
    ref = oracle.linear(inputs[-1][0], W, d, bias, wbits=8, exact_blas=True)
    Wq_h, _ = w.export()
    gu.assert_codes_close(Xq.cpu().numpy(), ref["Xq"], "Xq (graph replay)")
    gu.assert_codes_close(Wq_h, ref["Wq"], "Wq (graph replay)")
    gu.assert_y_close(gu.bf16_to_host(Y), ref["Y"], "Y (graph replay, oracle end to end)")
    w.close()


@pytest.mark.parametrize("wbits", [8, 4])
def test_rotate_quant_warm_read_changes_nothing(oracle, wbits):
    """The pass that also reads the next product's weights gives the bits of the plain pass and
    leaves the weights alone."""
    say(f"rotate_quant with the warming read, wbits={wbits}")
    M, K, N = 300, 1152, 400
    Xb, W, d, _ = wl.small_case(31, M, K, N, n_outliers=8)
    w = trdq.prepare_weights(gu.f32_to_dev(W), gu.f32_to_dev(d), wbits=wbits)
    before = w.export()
    X, dd = gu.bf16_to_dev(Xb), gu.f32_to_dev(d)
    out = []
    for warm in (None, w):
        Xq = torch.full((M, K), 99, dtype=torch.int8, device="cuda")
        sx = torch.full((M,), -1.0, dtype=torch.float32, device="cuda")
        trdq.rotate_quant(X, dd, Xq, sx, warm=warm)
        torch.cuda.synchronize()
        out.append((Xq, sx))
    assert torch.equal(out[0][0], out[1][0]) and torch.equal(out[0][1], out[1][1])
    after = w.export()
    assert np.array_equal(before[0], after[0]) and np.array_equal(before[1], after[1])
    w.close()


def test_shared_handles_on_two_streams(oracle):
    """The same prepared weights, rotation tables and layer used from two streams at once (handles are
    read-only after creation): every stream's outputs are the bits of the same calls issued one at a time."""
    say("two streams sharing the handles")
    M, K, N = 1024, 1152, 1152
    trdq.qgemm_set_variant(-1)
    cases = [wl.small_case(40 + i, M, K, N, n_outliers=8) for i in range(2)]
    _, W, d, bias = cases[0]
    dd, bd = gu.f32_to_dev(d), gu.f32_to_dev(bias)
    w = trdq.prepare_weights(gu.f32_to_dev(W), dd, wbits=8)
    Xs = [gu.bf16_to_dev(c[0]) for c in cases]
    ref_out = []
    for X in Xs:                                          # one at a time on the current stream
        Xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
        sx = torch.empty((M,), dtype=torch.float32, device="cuda")
        Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        trdq.rotate_quant(X, dd, Xq, sx, warm=w)
        trdq.qgemm(w, Xq, sx, Y, bias=bd)
        torch.cuda.synchronize()
        ref_out.append(Y)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    bufs = [(torch.empty((M, K), dtype=torch.int8, device="cuda"), torch.empty((M,), dtype=torch.float32, device="cuda"),
             torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")) for _ in range(2)]
    torch.cuda.synchronize()
    for rep in range(8):                                  # interleaved launches, no synchronisation in between
        for i in range(2):
            Xq, sx, Y = bufs[i]
            trdq.rotate_quant(Xs[i], dd, Xq, sx, stream=streams[i], warm=w)
            trdq.qgemm(w, Xq, sx, Y, bias=bd, stream=streams[i])
    torch.cuda.synchronize()
    for i in range(2):
        assert torch.equal(bufs[i][2], ref_out[i]), f"stream {i}"
    ref = oracle.linear(cases[1][0], W, d, bias, wbits=8, exact_blas=True)
    gu.assert_codes_close(bufs[1][0].cpu().numpy(), ref["Xq"], "Xq (second stream)")
    gu.assert_y_close(gu.bf16_to_host(bufs[1][2]), ref["Y"], "Y (second stream)")
    w.close()


def test_graph_replay_of_the_multi_kernel_calls():
    """The calls that launch several kernels and clear accumulators themselves (with fill kernels, not
    memsets) replay from a HIP graph: asymmetric pair, the two-pass dense-block pass, Eq. 11."""
    say("graph replay: asymmetric pair, wide dense pass, cosine similarity")
    M, K, N = 256, 1664, 144                   # 13 blocks: the block-resident, two-pass dense form
    inputs = [wl.small_case(50 + i, M, K, N, n_outliers=8) for i in range(3)]
    _, W, d, bias = inputs[0]
    dd, bb = gu.f32_to_dev(d), gu.f32_to_dev(bias)
    w = trdq.prepare_weights(gu.f32_to_dev(W), dd, wbits=8)
    Rs = wl.orthogonal_uniform_first_row(3, K // 128).astype(np.float32)
    rot = trdq.Rotation(gu.f32_to_dev(Rs.reshape(-1, 128)).view(-1, 128, 128), dd)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        X = gu.bf16_to_dev(inputs[0][0]).clone()
        Xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
        sx = torch.empty((M,), dtype=torch.float32, device="cuda")
        zc = torch.empty((M,), dtype=torch.int32, device="cuda")
        Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        Xq2 = torch.empty((M, K), dtype=torch.int8, device="cuda")
        sx2 = torch.empty((M,), dtype=torch.float32, device="cuda")
        ws = torch.zeros((3 * 4,), dtype=torch.float64, device="cuda")
        cs = torch.empty((4,), dtype=torch.float32, device="cuda")
        A4, B4 = X[:4], X[4:8]

        def calls():
            trdq.rotate_quant_asym(X, dd, Xq, sx, zc, stream=s)
            trdq.qgemm_asym(w, Xq, sx, zc, Y, bias=bb, stream=s)
            trdq.rotate_quant_dense(X, rot, Xq2, sx2, stream=s)
            trdq.cosine_similarity(A4, B4, ws, cs, stream=s)
        outs = (Xq, sx, zc, Y, Xq2, sx2, cs)
        calls()                               # warm-up outside the capture (one-time kernel attributes)
        s.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            calls()
        for Xb, _, _, _ in inputs:
            X.copy_(gu.bf16_to_dev(Xb))
            for t in outs:
                t.zero_()                     # host-launched work between the replays
            g.replay()
            s.synchronize()
            got = [t.clone() for t in outs]
            for t in outs:
                t.zero_()
            calls()
            s.synchronize()
            for a, b in zip(got, outs):
                if a.dtype == torch.float32 and a.numel() == 4:
                    assert torch.allclose(a, b, rtol=0, atol=1e-6)      # fp64 atomics: order may differ in the last bits
                else:
                    assert torch.equal(a, b)
    w.close(); rot.close()
