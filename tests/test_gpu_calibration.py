"""The two kernels of known traffic that byte counters and the dense scan's rate are held against: the copy copies,
the read reads every byte (its sink is written only where a wave's lanes each OR what they read to all ones) in every launch shape."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_copy_and_read_kernels():
    import paper_2309_13254_amd as zen

    zen.load_library()
    n = (1 << 22) + 4 * 37                                     # a ragged number of 16-byte vectors
    src = torch.randn(n, dtype=torch.float32, device="cuda")
    dst = torch.zeros_like(src)
    zen.zen_calibration_copy(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src.view(torch.int32), dst.view(torch.int32))
    even = torch.randint(-2**31, 2**31 - 1, (n,), dtype=torch.int64, device="cuda").to(torch.int32) & ~1
    shapes = [None, (256, 4, 4096, 0, 1), (512, 8, 128 << 10, 0, 0), (1024, 16, 1 << 20, 0, 1), (256, 8, 32 << 10, 64, 1),
              (1024, 4, 128 << 10, 7, 0)]
    for shape in shapes:
        sink = torch.zeros(64, dtype=torch.int32, device="cuda")
        zen.zen_calibration_read(even, sink, shape=shape)     # bit 0 is clear everywhere: no lane ORs to all ones, no store
        torch.cuda.synchronize()
        assert not sink.any().item(), shape
        ones = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        zen.zen_calibration_read(ones, sink, shape=shape)
        torch.cuda.synchronize()
        assert sink.any().item() and set(np.unique(sink.cpu().numpy()).tolist()) <= {0, -1}, shape
        sink.zero_()
        zen.zen_calibration_read(ones[: 4096], sink, shape=shape)              # a prefix shorter than one block
        torch.cuda.synchronize()
        assert sink.any().item(), shape
    with pytest.raises(zen.ZenError):
        zen.zen_calibration_read(src, sink, shape=(300, 8, 4096, 0, 1))       # no such block size
    with pytest.raises(zen.ZenError):
        zen.zen_calibration_read(src, sink, nbytes=24)                         # not a multiple of 16
