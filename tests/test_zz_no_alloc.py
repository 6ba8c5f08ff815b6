"""The entry point that allocates nothing (trdq_cosine_similarity_static: accumulators in a fixed
array inside the library) against the entry point that takes a workspace, through the C ABI: two
calls in a row, the second on a smaller input, so that what the first call left in the shared
array must not leak into the second."""
import numpy as np
import pytest
import torch

from paper_2503_06564_amd import trdq, workloads as wl
from gpu_util import dev

pytestmark = pytest.mark.gpu

TOL = 1e-5          # the bound of both entry points against the exact value (Eq. 11 in fp64 above 64 products)


def _inputs(n, L, seed):
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((n, L)).astype(np.float32)
    mix = rng.uniform(0.0, 1.0, (n, 1)).astype(np.float32)
    b = (mix * a + (1 - mix) * rng.standard_normal((n, L)).astype(np.float32)).astype(np.float32)
    ab, bb = wl.f32_to_bf16_bits(a), wl.f32_to_bf16_bits(b)
    to_dev = lambda bits: torch.from_numpy(bits.view(np.int16)).to(dev()).view(torch.bfloat16)
    return ab, bb, to_dev(ab), to_dev(bb)


def test_static_scratch_entry_point_matches_workspace_entry_point(oracle):
    for n, L, seed in ((300, 4096, 1), (7, 1000, 2)):                  # the second call is the smaller one
        print(f"cosine, no allocation: n={n} L={L}", flush=True)
        ab, bb, A, B = _inputs(n, L, seed)
        ws = torch.empty((3 * n,), dtype=torch.float64, device=dev())
        want_gpu = torch.full((n,), -9.0, dtype=torch.float32, device=dev())
        got = torch.full((n,), -9.0, dtype=torch.float32, device=dev())
        trdq.cosine_similarity(A, B, ws, want_gpu)
        trdq.cosine_similarity_static(A, B, got)
        torch.cuda.synchronize()
        # the two differ only in the order of the atomic float64 additions
        assert np.abs(got.cpu().numpy() - want_gpu.cpu().numpy()).max() <= 1e-6
        assert np.abs(got.cpu().numpy() - oracle.cosine_similarity(ab, bb)).max() <= TOL


def test_static_scratch_entry_point_rejects_too_many_segments():
    n = trdq.COSINE_STATIC_MAX_SEG + 1
    A = torch.zeros((n, 8), dtype=torch.bfloat16, device=dev())
    out = torch.zeros((n,), dtype=torch.float32, device=dev())
    with pytest.raises(trdq.TrdqError) as e:
        trdq.cosine_similarity_static(A, A, out)
    assert e.value.status == trdq.ERR_RANGE
    # the largest size it takes
    n = trdq.COSINE_STATIC_MAX_SEG
    A = torch.ones((n, 8), dtype=torch.bfloat16, device=dev())
    out = torch.zeros((n,), dtype=torch.float32, device=dev())
    trdq.cosine_similarity_static(A, A, out)
    torch.cuda.synchronize()
    assert bool((out == 1.0).all())
