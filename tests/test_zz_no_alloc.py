"""ff_crc32c_noalloc, the entry point for callers that cannot allocate (its scratch is a fixed
array in the library's device image), against ff_crc32c, the entry point it is a variant of, and
against the oracle: bit-exact, on calls in a row that share the array, the later ones smaller."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2512_03644_amd import binding as ff

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _crc_both(L, buf, nbytes):
    """(noalloc result, ff_crc32c result) for the first nbytes of buf, through the C ABI."""
    out = torch.full((2,), -1, dtype=torch.int32, device=DEV)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = L.ff_crc32c_noalloc(buf.data_ptr(), nbytes, out.data_ptr(), stream)
    assert rc == ff.FF_OK, ff.ff_strerror(rc)
    rc = L.ff_crc32c(buf.data_ptr(), nbytes, out.data_ptr() + 4, stream)
    assert rc == ff.FF_OK, ff.ff_strerror(rc)
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint32)
    return int(got[0]), int(got[1])


def test_noalloc_crc_matches_the_allocating_entry_point(oracle):
    L = ff.lib()
    g = torch.Generator(device=DEV)
    g.manual_seed(736)
    big = 37 * (1 << 20) + 5 * 1024 + 13       # 38 tiles of 1 MiB, the last one ragged, plus a tail
    buf = torch.randint(0, 256, (big,), dtype=torch.uint8, device=DEV, generator=g)
    host = buf.cpu().numpy()
    # two calls in a row, the second with a smaller input: the registers the first call left in
    # the shared array beyond the second call's tiles must not leak into its result
    for nbytes in (big, 3 * (1 << 20) + 1024 + 7, 1 << 20, 1023, 0, big):
        a, b = _crc_both(L, buf, nbytes)
        assert a == b == oracle.crc32c(host[:nbytes]), nbytes


def test_noalloc_crc_back_to_back_without_synchronising(oracle):
    """Calls on one stream may follow each other with no synchronisation in between."""
    L = ff.lib()
    g = torch.Generator(device=DEV)
    g.manual_seed(737)
    sizes = [9 * (1 << 20) + 77, 2 * (1 << 20), 5 * (1 << 20) + 4096, 16, 4 * (1 << 20) - 1]
    bufs = [torch.randint(0, 256, (max(n, 16),), dtype=torch.uint8, device=DEV, generator=g)
            for n in sizes]
    out = torch.full((len(sizes),), -1, dtype=torch.int32, device=DEV)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for k, (b, n) in enumerate(zip(bufs, sizes)):
        assert L.ff_crc32c_noalloc(b.data_ptr(), n, out.data_ptr() + 4 * k, stream) == ff.FF_OK
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint32)
    for k, (b, n) in enumerate(zip(bufs, sizes)):
        assert int(got[k]) == oracle.crc32c(b.cpu().numpy()[:n]), n


def test_noalloc_crc_rejects_what_does_not_fit():
    L = ff.lib()
    buf = torch.zeros(1024, dtype=torch.uint8, device=DEV)
    out = torch.full((1,), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
    # beyond the fixed capacity: refused before anything is enqueued (the size is only compared)
    rc = L.ff_crc32c_noalloc(buf.data_ptr(), ff.FF_CRC32C_NOALLOC_MAX_BYTES + 1, out.data_ptr(), None)
    assert rc == ff.FF_ERR_TOO_LARGE
    assert "scratch" in ff.ff_strerror(rc)
    assert L.ff_crc32c_noalloc(buf.data_ptr() + 1, 8, out.data_ptr(), None) == ff.FF_ERR_INVALID
    assert L.ff_crc32c_noalloc(buf.data_ptr(), 8, None, None) == ff.FF_ERR_NULL
    torch.cuda.synchronize()
    assert int(out.item()) == 0x5A5A5A5A
