"""Seeded synthetic inputs for the rotated-linear workloads (input data only).

This module holds none of the method's arithmetic: it draws activations,
weights, diagonal scales and biases with the shapes and value structure of a
DiT-XL/2-shaped denoiser (hidden 1152, MLP 4608) and of the paper's
observation that a few fixed channels carry massive, time-step dependent
outliers (Sec. 3.2, "Massive Outliers"; "Time-Steps Awareness Quantization").
Both the CPU oracle's tests and the GPU tests/benchmark take their inputs from
here, so the two sides see identical bits.  The real PixArt-alpha / Open-Sora
activations the paper measures on need model weights and datasets that are
not available; these generators stand in for them.

Every array is a pure function of (config id, layer kind, block, group/step):
numpy's PCG64 seeded with SeedSequence([tag, cfg, kind, block, index]).
Activations are rounded float32 -> bf16 (ties to even) and returned as uint16
bit patterns.
"""
from dataclasses import dataclass

import numpy as np

HIDDEN = 1152
BLOCK = 128

# (K, N) per layer kind of one DiT block
LAYER_SHAPES = {
    "qkv": (1152, 3456),
    "proj": (1152, 1152),
    "fc1": (1152, 4608),
    "fc2": (4608, 1152),
}
_KIND_ID = {"qkv": 0, "proj": 1, "fc1": 2, "fc2": 3}
_TAG_X, _TAG_W, _TAG_D, _TAG_B, _TAG_CH, _TAG_OS = 11, 12, 13, 14, 15, 16


@dataclass(frozen=True)
class Config:
    cfg: int
    name: str
    M: int                 # tokens
    kinds: tuple           # layer kinds present
    n_steps: int
    n_groups: int
    wbits: tuple           # weight widths exercised
    n_blocks: int          # distinct weight sets per kind
    outliers_per_1152: int


CONFIGS = (
    Config(0, "single_w8a8_512x1152x1152", 512, ("proj",), 1, 1, (8,), 1, 8),
    Config(1, "dit_xl2_256px_w8a8_m4096", 4096, ("qkv", "proj", "fc1", "fc2"), 10, 10, (8,), 1, 8),
    Config(2, "dit_xl2_512px_w4a8_m16384", 16384, ("qkv", "proj", "fc1", "fc2"), 10, 10, (4,), 1, 8),
    Config(3, "video_dit_w8a8_w4a8_m32768", 32768, ("qkv", "proj", "fc1", "fc2"), 20, 5, (8, 4), 1, 16),
    Config(4, "dit_xl2_28blocks_50steps_w8a8_m8192", 8192, ("qkv", "proj", "fc1", "fc2"), 50, 10, (8,), 28, 8),
)


def _rng(tag, cfg, kind, block, index):
    return np.random.default_rng(np.random.SeedSequence([tag, cfg, _KIND_ID[kind], block, index]))


def f32_to_bf16_bits(x):
    """float32 array -> uint16 bf16 bit patterns, round to nearest, ties to even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def bf16_bits_to_f32(h):
    return (np.asarray(h, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def draw_group(config, step):
    """Which of the config's n_groups seeded draws (activations, outlier scale) a sampling step reads:
    steps are dealt to the draws in contiguous near-equal runs.  This is part of the input recipe only;
    the method's own step -> group table is the library's (trdq_table_*) and, separately, the oracle's."""
    return (step * config.n_groups) // config.n_steps


def outlier_channels(config, kind):
    """Fixed outlier channel indices of a layer kind (drawn once per config and kind)."""
    K = LAYER_SHAPES[kind][0]
    n = config.outliers_per_1152 * (K // HIDDEN)
    return np.sort(_rng(_TAG_CH, config.cfg, kind, 0, 0).choice(K, size=n, replace=False))


def outlier_scale(config, kind, step):
    """Magnitude multiplier of the outlier channels at a sampling step."""
    if config.cfg == 0:
        return 50.0
    if config.cfg == 3:
        return 20.0 + 80.0 * step / (config.n_steps - 1)
    g = draw_group(config, step)
    return float(_rng(_TAG_OS, config.cfg, kind, 0, g).uniform(10.0, 80.0))


def make_x(config, kind, step=0, M=None, rows=None):
    """Activations of one layer at one sampling step: uint16 bf16 bits [M, K].

    Within a config the draw depends on the step's group (cfg 3: on the step
    itself, because the outlier magnitude moves with the step).  `rows` selects
    a subset of row indices of the full-size tensor without changing values."""
    K = LAYER_SHAPES[kind][0]
    M = config.M if M is None else M
    index = step if config.cfg == 3 else draw_group(config, step)
    x = _rng(_TAG_X, config.cfg, kind, 0, index).standard_normal((M, K), dtype=np.float32)
    ch = outlier_channels(config, kind)
    x[:, ch] *= np.float32(outlier_scale(config, kind, step))
    if rows is not None:
        x = x[np.asarray(rows)]
    return f32_to_bf16_bits(x)


def make_w(config, kind, block=0):
    """Weights [K, N] float32 ~ N(0, sigma = 0.02), layout C_in x C_out."""
    K, N = LAYER_SHAPES[kind]
    w = _rng(_TAG_W, config.cfg, kind, block, 0).standard_normal((K, N), dtype=np.float32)
    return w * np.float32(0.02)


def make_diag(config, kind, group=0):
    """The group's per-channel scale d_g [K] float32: ones for cfg 0, else LogNormal(0, 0.3)."""
    K = LAYER_SHAPES[kind][0]
    if config.cfg == 0:
        return np.ones(K, dtype=np.float32)
    return _rng(_TAG_D, config.cfg, kind, 0, group).lognormal(0.0, 0.3, K).astype(np.float32)


def make_bias(config, kind, block=0):
    """Bias [N] float32 ~ N(0, 0.1)."""
    N = LAYER_SHAPES[kind][1]
    return (_rng(_TAG_B, config.cfg, kind, block, 0).standard_normal(N, dtype=np.float32)
            * np.float32(0.1))


def small_case(seed, M, K, N, n_outliers=2, outlier=50.0, with_diag=True):
    """A small free-shape case (for tile-tail and brute-force tests)."""
    r = np.random.default_rng(np.random.SeedSequence([99, seed, M, K, N]))
    x = r.standard_normal((M, K), dtype=np.float32)
    if n_outliers and M:
        x[:, r.choice(K, size=min(n_outliers, K), replace=False)] *= np.float32(outlier)
    w = r.standard_normal((K, N), dtype=np.float32) * np.float32(0.02)
    d = (r.lognormal(0.0, 0.3, K).astype(np.float32) if with_diag
         else np.ones(K, dtype=np.float32))
    b = r.standard_normal(N, dtype=np.float32) * np.float32(0.1)
    return f32_to_bf16_bits(x), w, d, b


def orthogonal_uniform_first_row(seed, n_mats, B=128):
    """The random orthogonal matrices the greedy rotation search draws (Sec. 3.2): float64
    [n_mats, B, B], each orthogonal with a first row of equal entries 1/sqrt(B).  Built from a
    seeded Gaussian matrix whose first column is replaced by ones, orthonormalised (QR), transposed."""
    r = np.random.default_rng(np.random.SeedSequence([77, seed, n_mats, B]))
    out = np.empty((n_mats, B, B), dtype=np.float64)
    for i in range(n_mats):
        g = r.standard_normal((B, B))
        g[:, 0] = 1.0
        q, rr = np.linalg.qr(g)
        q = q * np.sign(rr[0, 0])           # first column +1/sqrt(B) everywhere
        out[i] = q.T
    return out
