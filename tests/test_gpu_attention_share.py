"""GPU parity of the cosine similarity of Eq. 11 (attention sharing, Sec. 3.3) against the oracle."""
import numpy as np
import pytest
import torch

from paper_2503_06564_amd import trdq, workloads as wl
from gpu_util import dev

pytestmark = pytest.mark.gpu

# fp32 sums of at most 64 exact products, fp64 above: |error| <= 64 * 2^-24 (|A||B|) < 4e-6, plus the float32 result
TOL = 1e-5


def _run(a_bits, b_bits, L=None):
    n, Lp = a_bits.shape
    L = Lp if L is None else L
    A = torch.from_numpy(a_bits.view(np.int16)).to(dev()).view(torch.bfloat16)[:, :L]
    B = torch.from_numpy(b_bits.view(np.int16)).to(dev()).view(torch.bfloat16)[:, :L]
    ws = torch.full((3 * n,), 7.0, dtype=torch.float64, device=dev())      # the call clears it
    out = torch.full((n,), -9.0, dtype=torch.float32, device=dev())
    trdq.cosine_similarity(A, B, ws, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("n,L,Lp", [(1, 7, 8), (3, 4096, 4096), (28, 12345, 12352), (5, 64, 64), (2, 1 << 20, 1 << 20),
                                    (300, 1000, 1000)])
def test_cosine_similarity_matches_oracle(oracle, n, L, Lp):
    print(f"cosine n={n} L={L}", flush=True)
    rng = np.random.default_rng(n * 131 + L)
    a = rng.standard_normal((n, Lp)).astype(np.float32)
    mix = rng.uniform(0.0, 1.0, (n, 1)).astype(np.float32)              # from unrelated to nearly equal
    b = (mix * a + (1 - mix) * rng.standard_normal((n, Lp)).astype(np.float32)).astype(np.float32)
    if n > 2:
        b[1] = -a[1]
        a[2] = 0.0
    ab, bb = wl.f32_to_bf16_bits(a), wl.f32_to_bf16_bits(b)
    got = _run(ab, bb, L)
    want = oracle.cosine_similarity(ab[:, :L], bb[:, :L])
    assert np.abs(got - want).max() <= TOL, f"max error {np.abs(got - want).max():.2e}"
    if n > 2:
        assert abs(got[1] + 1.0) <= TOL and got[2] == 0.0


def test_cosine_similarity_attention_sized(oracle):
    # one DiT-XL/2 block's attention output for a batch of 16 images: 4096 tokens x 1152 channels
    rng = np.random.default_rng(9)
    a = rng.standard_normal((1, 4096 * 1152)).astype(np.float32)
    b = (a + 0.1 * rng.standard_normal(a.shape)).astype(np.float32)
    ab, bb = wl.f32_to_bf16_bits(a), wl.f32_to_bf16_bits(b)
    got = _run(ab, bb)
    want = oracle.cosine_similarity(ab, bb)
    assert abs(got[0] - want[0]) <= TOL
    assert 0.99 < got[0] < 1.0
