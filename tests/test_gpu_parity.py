"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, element by element
on small and ragged inputs.  Integer/byte work: bit-exact."""
import numpy as np
import pytest
import torch

from paper_2512_03644_amd import binding as ff
from paper_2512_03644_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _host_segments(shard):
    """Host copies of the shard's segments as numpy arrays (uint8 views of the raw bytes)."""
    if shard.arena is not None:
        arena = shard.arena.cpu().numpy()
        return [arena[o:o + n] for o, n in shard.spans], arena
    return [wl.to_numpy_bytes(t) for t in shard.segments], None


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


def _pack_and_compare(shard, oracle, tile_log2=0):
    plan = ff.plan_for_shard(shard, tile_log2=tile_log2)
    chunks, crcs, bad, n_bad = ff.alloc_outputs(plan, DEV)
    chunks.fill_(0xA5)                       # every byte must be written, zero tail included
    crcs.fill_(-1)
    ff.ff_pack(plan, chunks, crcs)
    torch.cuda.synchronize()
    host, _ = _host_segments(shard)
    want_buf, want_crcs = oracle.pack(host, shard.chunk_bytes, threads=8)
    assert plan.payload_bytes == sum(h.size for h in host)
    assert np.array_equal(chunks.cpu().numpy(), want_buf)
    assert np.array_equal(_u32(crcs), want_crcs)
    return plan, chunks, crcs, bad, n_bad, want_buf, want_crcs


def _poison_segments(shard):
    if shard.arena is not None:
        for o, n in shard.spans:
            shard.arena[o:o + n] = 0xA5
    else:
        for t in shard.segments:
            t.view(torch.uint8).fill_(0xA5)


def _restore_and_compare(shard, plan, chunks, crcs, bad, n_bad, want_buf):
    """Restore into poisoned tensors; every segment byte comes back, nothing else changes."""
    before = shard.arena.cpu().numpy().copy() if shard.arena is not None else None
    _poison_segments(shard)
    bad.fill_(7)
    n_bad.fill_(99)
    ff.ff_restore(plan, chunks, crcs, bad, n_bad)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0 and not bad.cpu().numpy().any()
    host, arena = _host_segments(shard)
    got = np.concatenate(host)
    assert np.array_equal(got, want_buf[:got.size])
    if before is not None:
        assert np.array_equal(arena, before)      # gaps between the segments are untouched


@pytest.mark.parametrize("nbytes", [0, 1, 15, 16, 17, 1023, 1024, 1025, 24 * 1024, 25 * 1024 + 7,
                                    (1 << 20) - 1024, 1 << 20, (1 << 20) + 1024,
                                    3 * (1 << 20) + 12345])
def test_crc32c_of_a_buffer(oracle, nbytes):
    g = torch.Generator(device=DEV)
    g.manual_seed(1000 + nbytes)
    buf = torch.randint(0, 256, (max(nbytes, 16),), dtype=torch.uint8, device=DEV, generator=g)
    out = torch.zeros(1, dtype=torch.int32, device=DEV)
    ff.ff_crc32c(buf, nbytes, out)
    assert int(_u32(out)[0]) == oracle.crc32c(buf.cpu().numpy()[:nbytes])


def test_crc32c_check_value(oracle):
    buf = torch.zeros(16, dtype=torch.uint8, device=DEV)
    buf[:9] = torch.tensor(list(b"123456789"), dtype=torch.uint8)
    out = torch.zeros(1, dtype=torch.int32, device=DEV)
    ff.ff_crc32c(buf, 9, out)
    assert int(_u32(out)[0]) == 0xE3069283


def test_tiny_config_pack_restore(oracle):
    shard = wl.config_tiny(DEV)
    state = _pack_and_compare(shard, oracle)
    _restore_and_compare(shard, *state[:6])


@pytest.mark.parametrize("chunk,tile_log2", [(1024, 0), (2048, 0), (4096, 10), (32768, 12),
                                             (1 << 16, 0), (1 << 20, 17), (1 << 22, 0)])
def test_param_shard_chunk_and_tile_sizes(oracle, chunk, tile_log2):
    numels = [int(x) for x in np.random.default_rng(chunk).integers(1, 40000, size=24)]
    shard = wl.param_shard("p", numels, chunk, 77, DEV, tiny_recipe=True)
    state = _pack_and_compare(shard, oracle, tile_log2)
    _restore_and_compare(shard, *state[:6])


@pytest.mark.parametrize("seed,mu,n", [(1, 3.0, 3000), (2, 6.0, 2000), (3, 9.0, 400)])
def test_ragged_unaligned_segments(oracle, seed, mu, n):
    # many tiny tensors (down to one element), 2-byte granularity, every misalignment
    lay = wl.fragmented_layout(seed=seed, n_tensors=n, mu=mu, sigma=2.0, max_numel=1 << 18)
    shard = wl.fragmented_shard(lay, 1 << 16, seed=seed, device=DEV)
    assert len({o % 16 for o, _ in shard.spans}) == 8
    state = _pack_and_compare(shard, oracle)
    _restore_and_compare(shard, *state[:6])


def test_single_element_segments(oracle):
    lay = [(1, 2, (2 * i) % 16) for i in range(3000)] + [(1, 4, (4 * i) % 16) for i in range(500)]
    shard = wl.fragmented_shard(lay, 1024, seed=9, device=DEV)
    state = _pack_and_compare(shard, oracle)
    _restore_and_compare(shard, *state[:6])


def test_corruption_is_flagged_exactly(oracle):
    numels = [int(x) for x in np.random.default_rng(5).integers(1000, 90000, size=40)]
    shard = wl.param_shard("c", numels, 1 << 16, 5, DEV, tiny_recipe=True)
    plan, chunks, crcs, bad, n_bad, want_buf, want_crcs = _pack_and_compare(shard, oracle)
    hits = wl.corrupt_chunks(plan.num_chunks, shard.chunk_bytes, seed=8, fraction=0.05)
    dirty = chunks.clone()
    for c, off, bit in hits:
        dirty[c * shard.chunk_bytes + off] ^= (1 << bit)
    _poison_segments(shard)
    ff.ff_restore(plan, dirty, crcs, bad, n_bad)
    torch.cuda.synchronize()
    want_bad, want_n = oracle.verify(dirty.cpu().numpy(), want_crcs, shard.chunk_bytes)
    assert want_n == len(hits)
    assert int(n_bad.item()) == want_n
    assert np.array_equal(_u32(bad), want_bad)
    # data of bad chunks is scattered too
    got = np.concatenate(_host_segments(shard)[0])
    assert np.array_equal(got, dirty.cpu().numpy()[:got.size])
    # a flipped bit in the CRC array flags its chunk; verify-only leaves the tensors alone
    crcs2 = crcs.clone()
    crcs2[3] ^= (1 << 9)
    _poison_segments(shard)
    ff.ff_restore(plan, chunks, crcs2, bad, n_bad, flags=ff.FF_RESTORE_VERIFY_ONLY)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 1 and int(bad[3].item()) == 1 and int(bad.sum().item()) == 1
    assert all(bool((t.view(torch.uint8) == 0xA5).all()) for t in shard.segments)


def test_device_call_argument_errors():
    a = torch.zeros(4096, dtype=torch.float32, device=DEV)
    plan = ff.ff_snapshot_plan([a], 4096)
    chunks, crcs, bad, n_bad = ff.alloc_outputs(plan, DEV)
    L = ff.lib()
    assert L.ff_pack(plan.handle, chunks.data_ptr() + 4, crcs.data_ptr(), None) == ff.FF_ERR_INVALID
    assert L.ff_pack(plan.handle, None, crcs.data_ptr(), None) == ff.FF_ERR_NULL
    assert L.ff_restore(plan.handle, chunks.data_ptr(), crcs.data_ptr(), bad.data_ptr(),
                        n_bad.data_ptr(), 8, None) == ff.FF_ERR_INVALID
    assert L.ff_crc32c(chunks.data_ptr() + 1, 10, crcs.data_ptr(), None) == ff.FF_ERR_INVALID


def test_pack_on_a_side_stream(oracle):
    shard = wl.param_shard("s", [5000, 70000, 333], 1 << 15, 4, DEV, tiny_recipe=True)
    plan = ff.plan_for_shard(shard)
    chunks, crcs, bad, n_bad = ff.alloc_outputs(plan, DEV)
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        ff.ff_pack(plan, chunks, crcs)          # picks up the current (side) stream
        ff.ff_restore(plan, chunks, crcs, bad, n_bad, flags=ff.FF_RESTORE_VERIFY_ONLY, stream=st)
    st.synchronize()
    want_buf, want_crcs = oracle.pack(_host_segments(shard)[0], shard.chunk_bytes)
    assert np.array_equal(chunks.cpu().numpy(), want_buf)
    assert np.array_equal(_u32(crcs), want_crcs) and int(n_bad.item()) == 0
