"""The measurement helpers move exactly the bytes they claim: the plain copy that
HBM counters are scaled by, and the sequential streaming kernel with a given
read:write mix (the yardstick the data kernels are compared with)."""
import numpy as np
import pytest
import torch

from paper_2605_10670_amd import binding

pytestmark = pytest.mark.gpu

SEED = np.array([1, 2, 3, 4], dtype=np.uint32)


def test_copy_moves_every_byte_and_nothing_else():
    rng = np.random.default_rng(7)
    n = 16 * 1000 + 16                      # not a multiple of the workgroup's 4 KiB
    src = torch.from_numpy(rng.integers(0, 256, n + 64, dtype=np.uint8)).cuda()
    dst = torch.full((n + 64,), 0xAB, dtype=torch.uint8, device="cuda")
    binding.calibration_copy(dst, src, n)
    torch.cuda.synchronize()
    got = dst.cpu().numpy()
    assert np.array_equal(got[:n], src.cpu().numpy()[:n])
    assert (got[n:] == 0xAB).all()


@pytest.mark.parametrize("reads,writes", [(1, 1), (1, 8), (8, 1), (8, 8)])
def test_stream_reads_and_writes_the_stated_planes(reads, writes):
    rng = np.random.default_rng(100 + reads * 10 + writes)
    vecs, stride_vecs = 1000 + 37, 1000 + 37 + 5         # ragged tail, padded planes
    src_h = rng.integers(0, 2**32, (8, stride_vecs, 4), dtype=np.uint32)
    src = torch.from_numpy(src_h.view(np.int32)).cuda()
    dst = torch.full((8, stride_vecs, 4), -1, dtype=torch.int32, device="cuda")
    binding.calibration_stream(dst, src, vecs * 16, stride_vecs * 16, reads, writes)
    torch.cuda.synchronize()
    got = dst.cpu().numpy().view(np.uint32)
    v = np.broadcast_to(SEED, (vecs, 4)).copy()
    for j in range(reads):
        v ^= src_h[j, :vecs]
    for j in range(8):
        if j < writes:
            assert np.array_equal(got[j, :vecs], v + np.uint32(j)), f"plane {j}"
            assert (got[j, vecs:] == 0xFFFFFFFF).all(), f"padding after plane {j}"
        else:
            assert (got[j] == 0xFFFFFFFF).all(), f"plane {j} must stay untouched"


def test_stream_argument_checks():
    a = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    b = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    for args in [(64, 64, 2, 1), (64, 64, 1, 3), (24, 32, 1, 1), (64, 48, 1, 1), (64, 72, 1, 1),
                 (-16, 64, 1, 1)]:
        with pytest.raises(binding.EepError) as ei:
            binding.calibration_stream(b, a, *args)
        assert ei.value.code == binding.ERR_INVALID_ARG, args
    binding.calibration_stream(b, a, 0, 64, 1, 8)          # nothing to do is not an error
    torch.cuda.synchronize()
    assert (b.cpu().numpy() == 0).all()
