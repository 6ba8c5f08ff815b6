"""The two yardstick kernels behind the "measured ceiling" figures: their results are fixed by
construction, so a kernel that skipped work would be caught here rather than flatter a roofline."""
import numpy as np
import pytest
import torch

from paper_2503_06564_amd import trdq
from gpu_util import dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("workgroups,waves,iters", [(1, 1, 1), (3, 5, 7), (256, 4, 1000), (512, 8, 33)])
def test_matrix_issue_yardstick_sums(workgroups, waves, iters):
    n = workgroups * waves * 64
    sink = torch.full((n + 64,), -5, dtype=torch.int32, device=dev())
    ops = trdq.peak_mfma_i8(sink, workgroups, waves, iters)
    torch.cuda.synchronize()
    got = sink.cpu().numpy()
    # ones times ones over 64 products, 8 accumulators of 4 elements per lane
    assert np.all(got[:n] == 8 * 4 * 64 * iters)
    assert np.all(got[n:] == -5)                      # nothing past the launch's lanes
    assert ops == workgroups * waves * iters * 8 * 2 * 16 * 16 * 64


@pytest.mark.parametrize("n", [8, 64, 8 * 12345, 4096 * 1152, 8 * (256 * 16 * 256) + 8 * 999])
def test_stream_yardstick_copies_low_bytes(n):
    rng = np.random.default_rng(n)
    bits = rng.integers(0, 1 << 16, n, dtype=np.uint16)
    src = torch.from_numpy(bits.view(np.int16)).to(dev())
    dst = torch.full((n + 16,), 77, dtype=torch.int8, device=dev())
    trdq.peak_stream(src, dst[:n])
    torch.cuda.synchronize()
    got = dst.cpu().numpy()
    assert np.array_equal(got[:n].view(np.uint8), (bits & 0xff).astype(np.uint8))
    assert np.all(got[n:] == 77)


def test_stream_yardstick_empty_is_a_no_op():
    assert trdq.lib().trdq_peak_stream(None, None, 0, None) == trdq.OK
