"""GPU parity at the full sizes of the five synthetic workloads, in the launch configuration
bench.py times (built-in tile choice).  The GPU processes every token; the oracle recomputes a
sample of tokens one by one (first and last tile rows plus random rows), every weight code and
scale, and properties that hold for all rows are checked on the whole output."""
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
    trdq.qgemm_set_variant(-1)


def sample_rows(M, seed, n_random=64, edge=24, panel=128):
    """First and last rows, random rows, and one random row of every 128-token panel, so that every
    token panel of the product's tile map (and every 16-token group offset within some panel) is hit."""
    r = np.random.default_rng(seed)
    n_panels = (M + panel - 1) // panel
    per_panel = np.minimum(np.arange(n_panels) * panel + r.integers(0, panel, size=n_panels), M - 1)
    rows = np.concatenate([np.arange(min(edge, M)), np.arange(max(0, M - edge), M),
                           r.integers(0, M, size=n_random), per_panel])
    return np.unique(rows)


def oracle_group(oracle, cfg, step):
    """The step's group from the oracle's own table (default partition), never from the product."""
    return int(oracle.table_default(cfg.n_steps, cfg.n_groups)[step])


def check_layer(oracle, cfg, kind, step, wbits, block=0, fused_too=True, Xb=None, every_row=False):
    """One linear of a workload at full M: unfused (and fused) GPU path vs the oracle, on sampled rows
    (every token panel holds one) or on every row."""
    K, N = wl.LAYER_SHAPES[kind]
    g = oracle_group(oracle, cfg, step)
    Xb = wl.make_x(cfg, kind, step) if Xb is None else Xb
    M = Xb.shape[0]
    W, d, bias = wl.make_w(cfg, kind, block), wl.make_diag(cfg, kind, g), wl.make_bias(cfg, kind, block)
    Wd, dd, bd = gu.f32_to_dev(W), gu.f32_to_dev(d), gu.f32_to_dev(bias)
    w = trdq.prepare_weights(Wd, dd, wbits=wbits)
    X = gu.bf16_to_dev(Xb)
    Xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
    sx = torch.empty((M,), dtype=torch.float32, device="cuda")
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    trdq.rotate_quant(X, dd, Xq, sx)
    trdq.qgemm(w, Xq, sx, Y, bias=bd)
    torch.cuda.synchronize()

    # properties over ALL tokens: every live token uses the full code range, scales positive
    amax = Xq.abs().amax(dim=1)
    live = sx > 0
    assert bool((amax[live] == 127).all()) and bool((amax[~live] == 0).all())
    assert bool(torch.isfinite(Y.float()).all())

    rows = np.arange(M) if every_row else sample_rows(M, 1000 * cfg.cfg + step)
    ref = oracle.linear(Xb[rows], W, d, bias, wbits=wbits, exact_blas=True)
    idx = torch.from_numpy(rows).cuda()
    Xq_h, sx_h = Xq[idx].cpu().numpy(), sx[idx].cpu().numpy()
    gu.assert_codes_close(Xq_h, ref["Xq"], f"{kind} Xq")
    gu.assert_scales_close(sx_h, ref["sx"], f"{kind} s_x")
    codes, scales = w.export()
    gu.assert_codes_close(codes, ref["Wq"], f"{kind} Wq")
    gu.assert_scales_close(scales, ref["sw"], f"{kind} s_w")
    masks = gu.narrow_code_masks(8, wbits, Xq_h, ref["Xq"], codes, ref["Wq"])
    worst = gu.assert_y_close(gu.bf16_to_host(Y[idx]), ref["Y"], f"{kind} Y", *masks)
    # accumulators bit-exact given the GPU's own codes (oracle's exact integer product on them), so the
    # outputs are one bf16 step from the oracle's epilogue on those codes
    acc = oracle.acc_exact_blas(Xq_h, codes, None if wbits == 8 else 128)
    y_same = oracle.dequant(acc, sx_h, scales, bias)
    gu.assert_y_same_codes(gu.bf16_to_host(Y[idx]), y_same, f"{kind} Y (same codes)")
    if wbits == 8 and trdq.qgemm_tiled_supported(w, M):
        # the block-tiled pair (what bench.py and trdq_layer_forward take for the large shapes): the same codes,
        # moved, and the same bits out, on every token
        Xt = torch.empty((trdq.xq_tiled_nbytes(M, K),), dtype=torch.int8, device="cuda")
        sxt = torch.empty((M,), dtype=torch.float32, device="cuda")
        Yt = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        back = torch.empty((M, K), dtype=torch.int8, device="cuda")
        trdq.rotate_quant_tiled(X, dd, Xt, sxt, warm=w)
        trdq.qgemm_tiled(w, Xt, sxt, Yt, bias=bd)
        trdq.xq_untile(Xt, M, K, back)
        torch.cuda.synchronize()
        assert torch.equal(back, Xq) and torch.equal(sxt, sx), f"{kind}: tiled codes differ from row-major codes"
        assert torch.equal(Yt, Y), f"{kind}: tiled and row-major products differ"
    if fused_too:
        Yf = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        trdq.linear_fused(X, dd, w, Yf, bias=bd)
        torch.cuda.synchronize()
        # same arithmetic up to the rounding order of the rotation (see test_fused_matches_unfused_and_oracle)
        assert (Yf == Y).float().mean().item() >= 0.98, f"{kind}: fused and unfused outputs differ"
        gu.assert_y_close(gu.bf16_to_host(Yf[idx]), ref["Y"], f"{kind} Y fused", None, masks[1])
    w.close()
    return worst


def test_config0_single_layer_every_element(oracle):
    cfg = wl.CONFIGS[0]
    say("config 0: 512 x 1152 x 1152, every element")
    Xb, W = wl.make_x(cfg, "proj"), wl.make_w(cfg, "proj")
    d, bias = wl.make_diag(cfg, "proj"), wl.make_bias(cfg, "proj")
    ref = oracle.linear(Xb, W, d, bias, wbits=8)          # the plain int32 loop, all rows
    w = trdq.prepare_weights(gu.f32_to_dev(W), gu.f32_to_dev(d), wbits=8)
    Xq, sx = gu.gpu_rotate_quant(Xb, d)
    Y, acc = gu.gpu_qgemm(w, Xq, sx, bias, 1152, debug=True)
    gu.assert_codes_close(Xq.cpu().numpy(), ref["Xq"], "Xq")
    gu.assert_scales_close(sx.cpu().numpy(), ref["sx"], "s_x")
    codes, scales = w.export()
    gu.assert_codes_close(codes, ref["Wq"], "Wq")
    assert np.array_equal(acc.cpu().numpy(), oracle.igemm(Xq.cpu().numpy(), codes))
    gu.assert_y_close(gu.bf16_to_host(Y), ref["Y"], "Y")
    # the method's own claim on this input: rotated quantisation beats the exact product by ~1 %
    exact = wl.bf16_bits_to_f32(Xb).astype(np.float64) @ W.astype(np.float64) + bias
    got = gu.bits_to_f64(gu.bf16_to_host(Y))
    assert np.linalg.norm(got - exact) / np.linalg.norm(exact) < 0.02


@pytest.mark.parametrize("kind", ["qkv", "proj", "fc1", "fc2"])
@pytest.mark.parametrize("step", [0, 7])
def test_config1_dit_block_w8a8(oracle, kind, step):
    """The headline workload: every code, scale and output of all 4096 tokens against the oracle."""
    say(f"config 1: M=4096 {kind} step {step}, every element")
    check_layer(oracle, wl.CONFIGS[1], kind, step, 8, every_row=True)


@pytest.mark.parametrize("kind", ["qkv", "proj", "fc1", "fc2"])
def test_config2_w4a8_16384_tokens(oracle, kind):
    say(f"config 2: M=16384 W4A8 {kind}")
    check_layer(oracle, wl.CONFIGS[2], kind, 3, 4)


@pytest.mark.parametrize("kind", ["qkv", "proj", "fc1", "fc2"])
@pytest.mark.parametrize("step", [0, 19])
def test_config3_video_32768_tokens(oracle, kind, step):
    cfg = wl.CONFIGS[3]
    say(f"config 3: M=32768 {kind} step {step} (W8A8 and W4A8)")
    Xb = wl.make_x(cfg, kind, step)
    check_layer(oracle, cfg, kind, step, 8, Xb=Xb, fused_too=(kind != "fc2"))
    check_layer(oracle, cfg, kind, step, 4, Xb=Xb, fused_too=False)


def test_step_tables_match_the_oracle(oracle):
    """20 steps -> 5 groups (config 3), 50 -> 10 (config 4), 10 -> 10, and uneven cases."""
    for n_steps, n_groups in ((20, 5), (50, 10), (10, 10), (1, 1), (7, 3), (1000, 7)):
        t = trdq.Table(n_steps, n_groups)
        assert [t.lookup(s) for s in range(n_steps)] == [int(v) for v in oracle.table_default(n_steps, n_groups)]


@pytest.mark.parametrize("block,step", [(0, 0), (13, 27), (27, 49)])
@pytest.mark.parametrize("kind", ["qkv", "proj", "fc1", "fc2"])
def test_config4_denoiser_sweep_layers(oracle, block, step, kind):
    say(f"config 4: M=8192 block {block} {kind} step {step}")
    check_layer(oracle, wl.CONFIGS[4], kind, step, 8, block=block, fused_too=(block == 13 and kind == "proj"))


# every time-step group of the sweep (50 steps -> 10 groups: one step from each), one more block
@pytest.mark.parametrize("step", [2, 7, 12, 17, 22, 27, 32, 37, 42, 47])
@pytest.mark.parametrize("kind", ["qkv", "proj", "fc1", "fc2"])
def test_config4_every_time_step_group(oracle, step, kind):
    say(f"config 4: M=8192 block 7 {kind} step {step}")
    assert int(oracle.table_default(50, 10)[step]) == step // 5
    check_layer(oracle, wl.CONFIGS[4], kind, step, 8, block=7)


# ---- the full transform of Eq. 9 (rotation, zigzag permutation, rotation) at workload sizes ----

@pytest.mark.parametrize("cfg_id,kind,step", [(1, "fc1", 0), (1, "fc2", 7), (3, "proj", 19), (3, "fc2", 0)])
def test_rpr_full_size_sampled_rows(oracle, cfg_id, kind, step):
    cfg = wl.CONFIGS[cfg_id]
    say(f"config {cfg_id}: R P R {kind} step {step}, M={cfg.M}")
    K, N = wl.LAYER_SHAPES[kind]
    g = oracle_group(oracle, cfg, step)
    Xb = wl.make_x(cfg, kind, step)
    M = Xb.shape[0]
    W, d, bias = wl.make_w(cfg, kind), wl.make_diag(cfg, kind, g), wl.make_bias(cfg, kind)
    rows = sample_rows(M, 77 * cfg_id + step)
    # permutation from the once-rotated sample (a calibration set, as the paper builds P from activations)
    mag = np.abs(oracle.rotate(Xb[rows], d, 128)).max(axis=0).astype(np.float32)
    perm = trdq.zigzag_permutation(mag)
    assert np.array_equal(perm, oracle.zigzag(mag.astype(np.float64), 128))
    perm_d = torch.from_numpy(perm).cuda()
    Wd, dd, bd = gu.f32_to_dev(W), gu.f32_to_dev(d), gu.f32_to_dev(bias)
    w = trdq.prepare_weights_rpr(Wd, dd, perm_d, wbits=8)
    X = gu.bf16_to_dev(Xb)
    Xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
    sx = torch.empty((M,), dtype=torch.float32, device="cuda")
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    trdq.rotate_quant_rpr(X, dd, perm_d, Xq, sx, warm=w)
    trdq.qgemm(w, Xq, sx, Y, bias=bd)
    torch.cuda.synchronize()

    amax = Xq.abs().amax(dim=1)
    live = sx > 0
    assert bool((amax[live] == 127).all()) and bool((amax[~live] == 0).all())
    assert bool(torch.isfinite(Y.float()).all())

    ref = oracle.linear_rpr(Xb[rows], W, d, perm, bias, 128, 8, exact_blas=True)
    idx = torch.from_numpy(rows).cuda()
    gu.assert_codes_close(Xq[idx].cpu().numpy(), ref["Xq"], f"{kind} Xq (R P R)")
    gu.assert_scales_close(sx[idx].cpu().numpy(), ref["sx"], f"{kind} s_x (R P R)")
    codes, scales = w.export()
    gu.assert_codes_close(codes, ref["Wq"], f"{kind} Wq (R P R)")
    gu.assert_scales_close(scales, ref["sw"], f"{kind} s_w (R P R)")
    gu.assert_y_close(gu.bf16_to_host(Y[idx]), ref["Y"], f"{kind} Y (R P R)")
    w.close()


# ---- asymmetric activations, W6A6 and dense rotation blocks at workload sizes (sampled rows) ----

@pytest.mark.parametrize("cfg_id,kind,step", [(1, "qkv", 0), (1, "proj", 3), (1, "fc1", 7), (1, "fc2", 7), (3, "fc1", 19)])
def test_asym_full_size_sampled_rows(oracle, cfg_id, kind, step):
    cfg = wl.CONFIGS[cfg_id]
    say(f"config {cfg_id}: asymmetric activations {kind} step {step}, M={cfg.M}")
    K, N = wl.LAYER_SHAPES[kind]
    g = oracle_group(oracle, cfg, step)
    Xb = wl.make_x(cfg, kind, step)
    M = Xb.shape[0]
    W, d, bias = wl.make_w(cfg, kind), wl.make_diag(cfg, kind, g), wl.make_bias(cfg, kind)
    dd = gu.f32_to_dev(d)
    w = trdq.prepare_weights(gu.f32_to_dev(W), dd, wbits=8)
    Xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
    sx = torch.empty((M,), dtype=torch.float32, device="cuda")
    zc = torch.empty((M,), dtype=torch.int32, device="cuda")
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    trdq.rotate_quant_asym(gu.bf16_to_dev(Xb), dd, Xq, sx, zc, warm=w)
    trdq.qgemm_asym(w, Xq, sx, zc, Y, bias=gu.f32_to_dev(bias))
    torch.cuda.synchronize()
    # all tokens: both ends of the code range are used (the range contains zero), zero points in range
    assert bool((Xq.amax(dim=1)[sx > 0] == 127).all()) and bool((Xq.amin(dim=1)[sx > 0] == -128).all())
    assert bool(((zc >= -127) & (zc <= 128)).all()) and bool(torch.isfinite(Y.float()).all())
    rows = sample_rows(M, 77 * cfg.cfg + step)
    idx = torch.from_numpy(rows).cuda()
    ref = oracle.linear_asym(Xb[rows], W, d, bias, exact_blas=True)
    q = Xq[idx].cpu().numpy().astype(np.int16) + 128
    z = 128 - zc[idx].cpu().numpy()
    gu.assert_asym_codes_close(q, z, ref["Xq"], ref["zx"], f"{kind} Xq (asymmetric)")
    gu.assert_scales_close(sx[idx].cpu().numpy(), ref["sx"], f"{kind} s_x (asymmetric)")
    codes, scales = w.export()
    gu.assert_codes_close(codes, ref["Wq"], f"{kind} Wq (asymmetric)")
    gu.assert_y_close(gu.bf16_to_host(Y[idx]), ref["Y"], f"{kind} Y (asymmetric)")
    # identical codes and zero points: the integer sums, then the epilogue, in float64
    acc = oracle.acc_asym_exact_blas(q.astype(np.uint8), z.astype(np.int32), codes)
    want = gu.bits_to_f64(oracle.dequant(acc, sx[idx].cpu().numpy(), scales, bias))
    got = gu.bits_to_f64(gu.bf16_to_host(Y[idx]))
    row = np.abs(want).max(axis=1, keepdims=True)
    assert np.all(np.abs(got - want) <= np.abs(want) * 2.0 ** -7 + row * 1e-5)
    w.close()


@pytest.mark.parametrize("kind", ["proj", "fc2"])
def test_w6a6_full_size_sampled_rows(oracle, kind):
    cfg = wl.CONFIGS[1]
    say(f"config 1: W6A6 {kind}, M={cfg.M}")
    K, N = wl.LAYER_SHAPES[kind]
    Xb = wl.make_x(cfg, kind, 2)
    M = Xb.shape[0]
    W, d, bias = wl.make_w(cfg, kind), wl.make_diag(cfg, kind, oracle_group(oracle, cfg, 2)), wl.make_bias(cfg, kind)
    dd = gu.f32_to_dev(d)
    w = trdq.prepare_weights(gu.f32_to_dev(W), dd, wbits=6)
    Xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
    sx = torch.empty((M,), dtype=torch.float32, device="cuda")
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    trdq.rotate_quant_bits(gu.bf16_to_dev(Xb), dd, Xq, sx, 6, warm=w)
    trdq.qgemm(w, Xq, sx, Y, bias=gu.f32_to_dev(bias))
    torch.cuda.synchronize()
    assert bool((Xq.abs().amax(dim=1)[sx > 0] == 31).all())
    rows = sample_rows(M, 55)
    idx = torch.from_numpy(rows).cuda()
    ref = oracle.linear(Xb[rows], W, d, bias, wbits=6, abits=6, exact_blas=True)
    gu.assert_codes_close(Xq[idx].cpu().numpy(), ref["Xq"], f"{kind} Xq (6 bits)")
    codes, scales = w.export()
    gu.assert_codes_close(codes, ref["Wq"], f"{kind} Wq (6 bits)")
    Xq_h = Xq[idx].cpu().numpy()
    gu.assert_y_close(gu.bf16_to_host(Y[idx]), ref["Y"], f"{kind} Y (W6A6)",
                      *gu.narrow_code_masks(6, 6, Xq_h, ref["Xq"], codes, ref["Wq"]))
    y_same = oracle.dequant(oracle.acc_exact_blas(Xq_h, codes), sx[idx].cpu().numpy(), scales, bias)
    gu.assert_y_same_codes(gu.bf16_to_host(Y[idx]), y_same, f"{kind} Y (W6A6, same codes)")
    w.close()


@pytest.mark.parametrize("cfg_id,kind", [(1, "proj"), (1, "fc2"), (3, "qkv")])
def test_dense_blocks_full_size_sampled_rows(oracle, cfg_id, kind):
    cfg = wl.CONFIGS[cfg_id]
    say(f"config {cfg_id}: dense rotation blocks {kind}, M={cfg.M}")
    K, N = wl.LAYER_SHAPES[kind]
    Xb = wl.make_x(cfg, kind, 1)
    M = Xb.shape[0]
    W, d, bias = wl.make_w(cfg, kind), wl.make_diag(cfg, kind, oracle_group(oracle, cfg, 1)), wl.make_bias(cfg, kind)
    Rs = wl.orthogonal_uniform_first_row(300 + K, K // 128).astype(np.float32)
    rot = trdq.Rotation(gu.f32_to_dev(Rs.reshape(-1, 128)).view(-1, 128, 128), gu.f32_to_dev(d))
    w = trdq.prepare_weights_dense(gu.f32_to_dev(W), rot, wbits=8)
    Xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
    sx = torch.empty((M,), dtype=torch.float32, device="cuda")
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    trdq.rotate_quant_dense(gu.bf16_to_dev(Xb), rot, Xq, sx)
    trdq.qgemm(w, Xq, sx, Y, bias=gu.f32_to_dev(bias))
    torch.cuda.synchronize()
    assert bool((Xq.abs().amax(dim=1)[sx > 0] == 127).all())
    rows = sample_rows(M, 66)
    idx = torch.from_numpy(rows).cuda()
    ref = oracle.linear_dense(Xb[rows], W, d, Rs, bias, exact_blas=True)
    gu.assert_codes_close(Xq[idx].cpu().numpy(), ref["Xq"], f"{kind} Xq (dense blocks)")
    gu.assert_scales_close(sx[idx].cpu().numpy(), ref["sx"], f"{kind} s_x (dense blocks)")
    codes, scales = w.export()
    gu.assert_codes_close(codes, ref["Wq"], f"{kind} Wq (dense blocks)")
    gu.assert_y_close(gu.bf16_to_host(Y[idx]), ref["Y"], f"{kind} Y (dense blocks)")
    w.close(); rot.close()


def test_two_million_tokens_64_bit_offsets(oracle):
    """2 000 037 tokens x 1152 channels: byte offsets beyond 2^32 in X, element offsets beyond 2^31 in Xq;
    sampled rows (first and last tiles, random ones) against the oracle, properties over all tokens."""
    M, K, N = 2_000_037, 1152, 144
    say(f"large M: {M} x {K} -> {N}")
    gen = torch.Generator(device="cuda").manual_seed(5)
    X = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    for r0 in range(0, M, 262144):                       # in pieces: no float32 copy of the whole matrix
        r1 = min(M, r0 + 262144)
        X[r0:r1] = torch.randn((r1 - r0, K), generator=gen, device="cuda").to(torch.bfloat16)
    X[:, 100] *= 40.0                                    # an outlier channel
    _, W, d, bias = wl.small_case(91, 1, K, N)
    dd = gu.f32_to_dev(d)
    w = trdq.prepare_weights(gu.f32_to_dev(W), dd, wbits=8)
    Xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
    sx = torch.empty((M,), dtype=torch.float32, device="cuda")
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    trdq.rotate_quant(X, dd, Xq, sx, warm=w)
    trdq.qgemm(w, Xq, sx, Y, bias=gu.f32_to_dev(bias))
    torch.cuda.synchronize()
    assert bool((Xq.abs().amax(dim=1) == 127).all()) and bool((sx > 0).all())
    rows = sample_rows(M, 123, n_random=96, edge=40)
    idx = torch.from_numpy(rows).cuda()
    Xb = X[idx].view(torch.int16).cpu().numpy().view(np.uint16)
    ref = oracle.linear(Xb, W, d, bias, wbits=8, exact_blas=True)
    gu.assert_codes_close(Xq[idx].cpu().numpy(), ref["Xq"], "Xq (2M tokens)")
    gu.assert_scales_close(sx[idx].cpu().numpy(), ref["sx"], "s_x (2M tokens)")
    codes, _ = w.export()
    gu.assert_y_close(gu.bf16_to_host(Y[idx]), ref["Y"], "Y (2M tokens)")
    w.close()


# Both rotations dense (Eq. 10 as printed) at config 1's sizes: K = 1152 takes the 16-token kernel, K = 4608 the
# 8-token one and, with a workspace, the block-resident kernels; sampled rows against the oracle (the rotation acts on a row alone, the weights are exact).
@pytest.mark.parametrize("kind", ["proj", "fc2"])
def test_dense_chain_full_size_sampled_rows(oracle, kind):
    cfg = wl.CONFIGS[1]
    say(f"config 1: dense R1 P R2 {kind}, M={cfg.M}")
    K, N = wl.LAYER_SHAPES[kind]
    Xb = wl.make_x(cfg, kind, 2)
    M = Xb.shape[0]
    W, d, bias = wl.make_w(cfg, kind), wl.make_diag(cfg, kind, oracle_group(oracle, cfg, 2)), wl.make_bias(cfg, kind)
    R1 = wl.orthogonal_uniform_first_row(500 + K, K // 128).astype(np.float32)
    R2 = wl.orthogonal_uniform_first_row(600 + K, K // 128).astype(np.float32)
    rot1 = trdq.Rotation(gu.f32_to_dev(R1.reshape(-1, 128)).view(-1, 128, 128), gu.f32_to_dev(d))
    rot2 = trdq.Rotation(gu.f32_to_dev(R2.reshape(-1, 128)).view(-1, 128, 128))
    # the permutation is an input of both sides: dealt by the oracle from its own once-rotated activations
    perm = oracle.zigzag(np.abs(oracle.rotate_dense(Xb, d, R1)).max(axis=0), 128).astype(np.int32)
    perm_dev = torch.from_numpy(perm).cuda()
    w = trdq.prepare_weights_dense_rpr(gu.f32_to_dev(W), rot1, perm_dev, rot2, wbits=8)
    Xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
    sx = torch.empty((M,), dtype=torch.float32, device="cuda")
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    trdq.rotate_quant_dense_rpr(gu.bf16_to_dev(Xb), rot1, perm_dev, rot2, Xq, sx)
    trdq.qgemm(w, Xq, sx, Y, bias=gu.f32_to_dev(bias))
    torch.cuda.synchronize()
    assert bool((Xq.abs().amax(dim=1)[sx > 0] == 127).all())
    rows = sample_rows(M, 66)
    idx = torch.from_numpy(rows).cuda()
    ref = oracle.linear_dense_rpr(Xb[rows], W, d, R1, perm, R2, bias, exact_blas=True)
    gu.assert_codes_close(Xq[idx].cpu().numpy(), ref["Xq"], f"{kind} Xq (dense R1 P R2)")
    gu.assert_scales_close(sx[idx].cpu().numpy(), ref["sx"], f"{kind} s_x (dense R1 P R2)")
    codes, scales = w.export()
    gu.assert_codes_close(codes, ref["Wq"], f"{kind} Wq (dense R1 P R2)")
    gu.assert_y_close(gu.bf16_to_host(Y[idx]), ref["Y"], f"{kind} Y (dense R1 P R2)")
    # the workspace form (block-resident kernels; for K = 1152 it needs none and is the call above)
    nbytes = trdq.rotate_quant_dense_rpr_ws_nbytes(M, K)
    assert (nbytes > 0) == (K > 1536)
    ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda") if nbytes else None
    Xq2 = torch.full((M, K), 99, dtype=torch.int8, device="cuda")
    sx2 = torch.full((M,), -1.0, dtype=torch.float32, device="cuda")
    trdq.rotate_quant_dense_rpr_ws(gu.bf16_to_dev(Xb), rot1, perm_dev, rot2, Xq2, sx2, ws)
    torch.cuda.synchronize()
    assert bool((Xq2.abs().amax(dim=1)[sx2 > 0] == 127).all())
    gu.assert_codes_close(Xq2[idx].cpu().numpy(), ref["Xq"], f"{kind} Xq (dense R1 P R2, workspace)")
    gu.assert_scales_close(sx2[idx].cpu().numpy(), ref["sx"], f"{kind} s_x (dense R1 P R2, workspace)")
    # the two forms against each other on every token: the same maxima to rounding, codes one step apart at most
    assert torch.allclose(sx2, sx, rtol=1e-5, atol=0)
    dq = (Xq2.int() - Xq.int()).abs()
    assert int(dq.max()) <= 1 and float((dq > 0).float().mean()) <= 1e-4
    w.close(); rot1.close(); rot2.close()
