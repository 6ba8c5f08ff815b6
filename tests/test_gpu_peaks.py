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


def _h(x):
    x = x.astype(np.uint64) & 0xFFFFFFFF
    x ^= x >> 16
    x = (x * 0x7feb352d) & 0xFFFFFFFF
    x ^= x >> 15
    x = (x * 0x846ca68b) & 0xFFFFFFFF
    x ^= x >> 16
    return x.astype(np.uint32)


@pytest.mark.parametrize("workgroups,waves,iters", [(1, 1, 1), (2, 8, 5), (256, 4, 300)])
def test_matrix_issue_yardstick_on_random_bytes(workgroups, waves, iters):
    """The random-operand kernel against the matrix instruction written out on the host: A is 16 x 64
    (row = lane % 16, bytes 16 (lane / 16) .. + 15 of the row in the lane), B is 64 x 16 the same way
    (column = lane % 16), and lane l ends with D[4 (l / 16) .. + 3][l % 16]."""
    n = workgroups * waves * 64
    sink = torch.full((n + 64,), -5, dtype=torch.int32, device=dev())
    ops = trdq.peak_mfma_i8(sink, workgroups, waves, iters, random_data=True)
    torch.cuda.synchronize()
    got = sink.cpu().numpy()
    assert ops == workgroups * waves * iters * 8 * 2 * 16 * 16 * 64
    t = np.arange(waves * 64, dtype=np.uint64)

    def frags(mul, imul, jmul, add, count):
        out = []
        for i in range(count):
            words = np.stack([_h(t * mul + i * imul + j * jmul + add) for j in range(4)], axis=1)   # [threads, 4]
            out.append(words.view(np.int8).reshape(waves, 64, 16).astype(np.int64))               # little-endian bytes
        return out
    A, B = frags(977, 31, 7, 1, 2), frags(131, 17, 3, 5, 4)
    want = np.zeros((waves, 64), dtype=np.int64)
    for w_ in range(waves):
        def matrix(f):       # [16 rows/cols][64 k] from the lanes of wave w_
            return f[w_].reshape(4, 16, 16).transpose(1, 0, 2).reshape(16, 64)
        for k in range(8):
            D = matrix(A[k & 1]) @ matrix(B[k >> 1]).T                  # [16 i][16 j]
            per_lane = D.reshape(4, 4, 16).sum(axis=1)                   # rows 4 g .. 4 g + 3 -> [g][j]
            want[w_] += per_lane.reshape(64)
    want = (want * iters).astype(np.int64)
    want32 = ((want + (1 << 31)) % (1 << 32) - (1 << 31)).astype(np.int32)
    assert np.array_equal(got[:n].reshape(workgroups, waves, 64), np.broadcast_to(want32, (workgroups, waves, 64)))
    assert np.all(got[n:] == -5)


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
