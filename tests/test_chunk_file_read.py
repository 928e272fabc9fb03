"""a3_chunk_file_read (host only: files -> host buffers): bytes against what was written, short files, bad
arguments.  No GPU."""
import ctypes as C
import os

import numpy as np
import pytest
import torch

from paper_2511_17560_amd import api


def _files(tmp_path, n, size, seed=0):
    rng = np.random.default_rng(seed)
    data, fds = [], []
    for i in range(n):
        b = rng.integers(0, 256, size=size + 1000 * i, dtype=np.uint8)
        p = tmp_path / f"chunk{i}.bin"
        p.write_bytes(b.tobytes())
        data.append(b)
        fds.append(os.open(p, os.O_RDONLY))
    return data, fds


@pytest.mark.parametrize("threads", [1, 3, 16, 100])
def test_blocks_land_byte_for_byte(tmp_path, threads):
    data, fds = _files(tmp_path, 7, 300_000)
    try:
        offs = [0, 17, 4096, 123_457, 0, 299_999, 5]
        lens = [300_000, 1, 100_000, 150_000, 0, 1, 250_000]
        dst = [torch.full((n + 3,), 7, dtype=torch.uint8) for n in lens]
        api.a3_chunk_file_read(fds, offs, lens, dst, n_threads=threads)
        for b, o, n, d in zip(data, offs, lens, dst):
            got = d.numpy()
            assert np.array_equal(got[:n], b[o:o + n]) and np.all(got[n:] == 7)      # nothing past the block is touched
        # the descriptors' own positions are not moved
        assert all(os.lseek(fd, 0, os.SEEK_CUR) == 0 for fd in fds)
        # the same block twice from one file, into two buffers
        a, b2 = torch.zeros(1000, dtype=torch.uint8), torch.zeros(1000, dtype=torch.uint8)
        api.a3_chunk_file_read([fds[0], fds[0]], [10, 10], [1000, 1000], [a, b2])
        assert torch.equal(a, b2) and np.array_equal(a.numpy(), data[0][10:1010])
    finally:
        for fd in fds:
            os.close(fd)


def test_errors(tmp_path):
    data, fds = _files(tmp_path, 2, 5000)
    try:
        buf = torch.zeros(10_000, dtype=torch.uint8)
        with pytest.raises(api.A3Error) as e:                    # the file ends inside the block
            api.a3_chunk_file_read([fds[0]], [4000], [2000], [buf])
        assert e.value.status == api.A3_ERR_IO and "block 0" in str(e.value)
        closed = os.open(tmp_path / "chunk0.bin", os.O_RDONLY)
        os.close(closed)
        with pytest.raises(api.A3Error) as e:                    # a descriptor that is not open
            api.a3_chunk_file_read([fds[1], closed], [0, 0], [100, 100], [buf, buf[200:]])
        assert e.value.status == api.A3_ERR_IO and "block 1" in str(e.value)
        L = api.lib()
        one = (C.c_int * 1)(fds[0])
        off, n, neg = (C.c_longlong * 1)(0), (C.c_size_t * 1)(10), (C.c_longlong * 1)(-1)
        ptr, null = (C.c_void_p * 1)(buf.data_ptr()), (C.c_void_p * 1)(None)
        assert L.a3_chunk_file_read(0, None, None, None, None, 1) == api.A3_OK
        assert L.a3_chunk_file_read(-1, one, off, n, ptr, 1) == api.A3_ERR_INVALID_ARG
        assert L.a3_chunk_file_read(1, None, off, n, ptr, 1) == api.A3_ERR_INVALID_ARG
        assert L.a3_chunk_file_read(1, one, neg, n, ptr, 1) == api.A3_ERR_INVALID_ARG
        assert L.a3_chunk_file_read(1, one, off, n, null, 1) == api.A3_ERR_INVALID_ARG
        assert L.a3_chunk_file_read(1, (C.c_int * 1)(-3), off, n, ptr, 1) == api.A3_ERR_INVALID_ARG
        assert L.a3_chunk_file_read(1, one, off, n, ptr, 0) == api.A3_OK                   # thread count is clamped
        assert L.a3_strerror(api.A3_ERR_IO) == b"file read failed"
    finally:
        for fd in fds:
            os.close(fd)
