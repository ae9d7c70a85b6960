"""The two measuring-stick kernels: a contiguous copy and a chunk-permuted copy.  They carry no part of
the method, but the roofline figures are read against them, so they must copy what they claim to."""
import numpy as np
import pytest

from paper_2408_08147_amd import kvx


def test_chunk_yardstick_argument_errors():
    E = kvx.KvxError
    for dst, src, nbytes, chunk, code in (
            (0, 4096, 8192, 4096, kvx.ERR_INVALID_ARG),
            (4096, 0, 8192, 4096, kvx.ERR_INVALID_ARG),
            (4096, 65536, 8192, 2048, kvx.ERR_INVALID_ARG),      # below 4 KiB
            (4096, 65536, 3 * 4096, 12288, kvx.ERR_INVALID_ARG),  # not a power of two
            (4096, 65536, 8192 + 4096, 8192, kvx.ERR_INVALID_ARG),  # does not divide
            (4096 + 8, 65536, 8192, 4096, kvx.ERR_ALIGNMENT),
            (4096, 1 << 40, 1 << 36, 4096, kvx.ERR_UNSUPPORTED)):
        with pytest.raises(E) as ei:
            kvx.kvx_copy_yardstick_chunks(dst, src, nbytes, chunk)
        assert ei.value.status == code, (dst, src, nbytes, chunk)


@pytest.mark.gpu
@pytest.mark.parametrize("chunk,n", [(4096, 1), (4096, 37), (8192, 129), (65536, 19), (1 << 20, 5)])
def test_chunk_yardstick_copies_through_both_permutations(chunk, n):
    import torch
    rng = np.random.default_rng(chunk + n)
    dev = torch.device("cuda:0")
    src = rng.integers(0, 256, size=chunk * n, dtype=np.uint8)
    ps, pd = rng.permutation(n).astype(np.uint32), rng.permutation(n).astype(np.uint32)
    s = src.reshape(n, chunk)
    stream = torch.cuda.Stream(device=dev)
    with torch.cuda.stream(stream):
        src_t = torch.from_numpy(src).to(dev)
        ps_t, pd_t = torch.from_numpy(ps).to(dev), torch.from_numpy(pd).to(dev)
        for a, b in ((None, None), (ps_t, None), (None, pd_t), (ps_t, pd_t)):
            dst_t = torch.full((chunk * n + 64,), 0xEE, dtype=torch.uint8, device=dev)
            kvx.kvx_copy_yardstick_chunks(dst_t.data_ptr(), src_t.data_ptr(), chunk * n, chunk,
                                          a.data_ptr() if a is not None else 0,
                                          b.data_ptr() if b is not None else 0, stream.cuda_stream)
            stream.synchronize()
            want = np.empty_like(s)
            want[pd if b is not None else np.arange(n)] = s[ps if a is not None else np.arange(n)]
            got = dst_t.cpu().numpy()
            assert np.array_equal(got[:chunk * n].reshape(n, chunk), want)
            assert (got[chunk * n:] == 0xEE).all()


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


@pytest.mark.gpu
def test_one_way_yardsticks():
    import torch
    dev = torch.device("cuda:0")
    n = 37 * 4096
    stream = torch.cuda.Stream(device=dev)
    with torch.cuda.stream(stream):
        buf = torch.full((n + 4096,), 0xEE, dtype=torch.uint8, device=dev)
        kvx.kvx_write_yardstick(buf.data_ptr(), n, 0x01020304, stream.cuda_stream)
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        kvx.kvx_read_yardstick(buf.data_ptr(), n, sink.data_ptr(), stream.cuda_stream)
    stream.synchronize()
    got = buf.cpu().numpy()
    assert np.array_equal(got[:n].view("<u4"), np.full(n // 4, 0x01020304, dtype="<u4"))
    assert (got[n:] == 0xEE).all()
    assert int(sink.item()) == 0


def test_one_way_yardstick_argument_errors():
    for fn, args, code in ((kvx.kvx_write_yardstick, (0, 4096, 1), kvx.ERR_INVALID_ARG),
                           (kvx.kvx_write_yardstick, (4096, 4095, 1), kvx.ERR_INVALID_ARG),
                           (kvx.kvx_write_yardstick, (4096 + 4, 4096, 1), kvx.ERR_ALIGNMENT),
                           (kvx.kvx_write_yardstick, (4096, 1 << 36, 1), kvx.ERR_UNSUPPORTED),
                           (kvx.kvx_read_yardstick, (4096, 4096, 0), kvx.ERR_INVALID_ARG),
                           (kvx.kvx_read_yardstick, (0, 4096, 64), kvx.ERR_INVALID_ARG),
                           (kvx.kvx_read_yardstick, (4096, 4096, 66), kvx.ERR_ALIGNMENT)):
        with pytest.raises(kvx.KvxError) as ei:
            fn(*args)
        assert ei.value.status == code, (fn.__name__, args)
