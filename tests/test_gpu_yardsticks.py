"""The measuring-stick kernel: a plain contiguous copy.  It carries no part of the method, but the roofline
figures and the counter calibration are read against it, so it must copy what it claims to."""
import numpy as np
import pytest

from paper_2408_08147_amd import kvx


@pytest.mark.gpu
@pytest.mark.parametrize("nbytes", [16, 4096 + 16, 3 * (1 << 20) + 48])
def test_plain_yardstick_copies(nbytes):
    import torch
    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream(device=dev)
    with torch.cuda.stream(stream):
        src_t = torch.randint(0, 256, (nbytes,), dtype=torch.int16, device=dev).to(torch.uint8)
        dst_t = torch.full((nbytes + 64,), 0xEE, dtype=torch.uint8, device=dev)
        kvx.kvx_copy_yardstick(dst_t.data_ptr(), src_t.data_ptr(), nbytes, stream.cuda_stream)
    stream.synchronize()
    assert torch.equal(dst_t[:nbytes], src_t)
    assert bool((dst_t[nbytes:] == 0xEE).all())
