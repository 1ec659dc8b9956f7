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


def _pack_and_compare(shard, oracle, tile_log2=0, flags=0):
    plan = ff.plan_for_shard(shard, flags=flags, tile_log2=tile_log2)
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


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_tiles_with_a_few_segment_boundaries(oracle, seed):
    # tensors of 4-40 KB at every 2-byte misalignment: most 32 KiB tiles hold 2-5 pieces
    lay = wl.fragmented_layout(seed=seed, n_tensors=1200, mu=8.6, sigma=0.6, max_numel=1 << 15)
    shard = wl.fragmented_shard(lay, 1 << 17, seed=seed, device=DEV)
    state = _pack_and_compare(shard, oracle)
    _restore_and_compare(shard, *state[:6])


def test_whole_tiles_at_every_offset_within_a_line(oracle):
    # tensors of 3-4 tiles each, ragged, starting at every even offset within a 128-byte line:
    # most tiles lie inside one tensor, at every misalignment of the tensor side (on restore
    # these are the tiles whose stores are lined up with the tensor)
    rng = np.random.default_rng(5)
    lay = [(int(rng.integers(48000, 60000)), 2, int(rng.integers(0, 8)) * 2) for _ in range(320)]
    shard = wl.fragmented_shard(lay, 1 << 18, seed=5, device=DEV)
    assert len({o % 128 for o, _ in shard.spans}) == 64
    state = _pack_and_compare(shard, oracle)
    _restore_and_compare(shard, *state[:6])


@pytest.mark.parametrize("tail", [2, 14, 16, 18, 1022, 1024, 1026, 16384 + 6, 32766])
def test_payload_end_inside_a_tile(oracle, tail):
    # three full tiles, then `tail` bytes split over segments of 2-byte granularity: the payload
    # ends inside the fourth tile at every kind of position (inside a lane, on a lane or row edge)
    lay = [(3 * 16384 + 5, 2, 2), (max(tail // 2 - 5, 0), 2, 6)]
    if tail // 2 - 5 < 0:
        lay = [(3 * 16384 + tail // 2, 2, 2)]
    shard = wl.fragmented_shard(lay, 1 << 17, seed=tail, device=DEV)
    assert shard.payload_bytes == 3 * 32768 + tail
    state = _pack_and_compare(shard, oracle)
    _restore_and_compare(shard, *state[:6])


@pytest.mark.parametrize("pieces", [2, 3, 4, 5, 6])
def test_boundaries_at_every_offset_in_a_lane(oracle, pieces):
    # one 32 KiB tile cut into `pieces` segments; the cuts walk through all eight halfword
    # positions of a lane, include segments shorter than a lane, and two cuts inside one lane
    lay, used = [], 0
    cuts = [1024 * 3 + 2 * k for k in range(8)][:pieces - 1]
    cuts = sorted(set(cuts + ([9000, 9002, 9006] if pieces >= 4 else [])))[:pieces - 1]
    for c in cuts + [32768]:
        lay.append(((c - used) // 2, 2, (2 * len(lay)) % 16))
        used = c
    lay.append((20000, 4, 4))                       # more tiles behind it
    shard = wl.fragmented_shard(lay, 1 << 16, seed=pieces, device=DEV)
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


@pytest.mark.parametrize("chunk,tile_log2", [(1 << 15, 0), (1 << 16, 0), (1 << 16, 12), (1 << 18, 0),
                                             (1 << 20, 14), (1 << 17, 17)])
def test_verify_only_every_tile_position(oracle, chunk, tile_log2):
    """A read-only pass folds several tiles as one; a flipped bit in any tile of a chunk, and at
    the first and last byte of a chunk, must flag exactly that chunk."""
    numels = [int(x) for x in np.random.default_rng(chunk + tile_log2).integers(20000, 200000, size=12)]
    shard = wl.param_shard("v", numels, chunk, 31, DEV, tiny_recipe=True)
    plan, chunks, crcs, bad, n_bad, want_buf, want_crcs = _pack_and_compare(shard, oracle, tile_log2)
    tile = 1 << (tile_log2 or 15)
    tile = min(tile, chunk)
    rng = np.random.default_rng(7)
    dirty = chunks.clone()
    hit = []
    for c in range(plan.num_chunks):
        k = c % (chunk // tile + 2)           # tile position inside the chunk; two extra cases
        if k == chunk // tile:
            off = 0
        elif k == chunk // tile + 1:
            off = chunk - 1
        else:
            off = k * tile + int(rng.integers(0, tile))
        if c % 3 != 2:                        # leave every third chunk clean
            dirty[c * chunk + off] ^= (1 << int(rng.integers(0, 8)))
            hit.append(c)
    _poison_segments(shard)
    ff.ff_restore(plan, dirty, crcs, bad, n_bad, flags=ff.FF_RESTORE_VERIFY_ONLY)
    torch.cuda.synchronize()
    want_bad, want_n = oracle.verify(dirty.cpu().numpy(), want_crcs, chunk)
    assert want_n == len(hit) and list(np.nonzero(want_bad)[0]) == hit
    assert int(n_bad.item()) == want_n
    assert np.array_equal(_u32(bad), want_bad)
    assert all(bool((t.view(torch.uint8) == 0xA5).all()) for t in shard.segments)
    # clean buffer: nothing flagged
    ff.ff_restore(plan, chunks, crcs, bad, n_bad, flags=ff.FF_RESTORE_VERIFY_ONLY)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0 and int(bad.sum().item()) == 0
    # skip-bad: chunks that verify are scattered, the others leave their ranges untouched
    _poison_segments(shard)
    ff.ff_restore(plan, dirty, crcs, bad, n_bad, flags=ff.FF_RESTORE_SKIP_BAD)
    torch.cuda.synchronize()
    assert np.array_equal(_u32(bad), want_bad)
    got = np.concatenate(_host_segments(shard)[0])
    clean = chunks.cpu().numpy()[:got.size]
    for c in range(plan.num_chunks):
        lo, hi = c * chunk, min((c + 1) * chunk, got.size)
        if want_bad[c]:
            assert bool((got[lo:hi] == 0xA5).all())
        else:
            assert np.array_equal(got[lo:hi], clean[lo:hi])


def test_empty_segments_and_exact_multiple_of_the_chunk(oracle):
    # empty tensors take no place in the stream; a payload that is a whole number of chunks has
    # no zero tail; a payload smaller than one chunk is one chunk, mostly zeros
    g = torch.Generator(device=DEV)
    g.manual_seed(11)
    mk = lambda n, dt: torch.randn(n, device=DEV, generator=g).to(dt)
    segs = [mk(0, torch.float32), mk(3 * 1024, torch.float32), mk(0, torch.bfloat16),
            mk(2 * 1024, torch.bfloat16), mk(0, torch.float32)]
    shard = wl.Shard("z", 4096, segs, [])
    state = _pack_and_compare(shard, oracle)
    plan = state[0]
    assert plan.payload_bytes == 16384 == plan.buffer_bytes and plan.num_segments == 2
    _restore_and_compare(shard, *state[:6])
    small = wl.Shard("y", 1 << 20, [mk(5, torch.bfloat16), mk(1, torch.float32)], [])
    state = _pack_and_compare(small, oracle)
    plan = state[0]
    assert plan.payload_bytes == 14 and plan.num_chunks == 1 and plan.buffer_bytes == 1 << 20
    _restore_and_compare(small, *state[:6])


def test_maximum_chunk_size(oracle):
    # 1 GiB chunks: two of them, the second mostly zero tail; the fused step crosses the boundary
    C = 1 << 30
    numels = [60 * (1 << 20) + 3, 20 * (1 << 20) + 1]           # 80 Mi elements, 1.17 GB
    shard, plan = _adam_and_compare(oracle, numels, C, seed=12)
    assert plan.num_chunks == 2 and plan.chunk_bytes == C
    chunks, crcs, bad, n_bad = ff.alloc_outputs(plan, DEV)
    ff.ff_pack(plan, chunks, crcs)
    saved = [t.clone() for t in shard.segments]
    _poison_segments(shard)
    chunks[C + 12345] ^= 4
    ff.ff_restore(plan, chunks, crcs, bad, n_bad)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 1 and bad.tolist() == [0, 1]
    chunks[C + 12345] ^= 4
    ff.ff_restore(plan, chunks, crcs, bad, n_bad)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0
    assert all(torch.equal(a.view(torch.uint8), b.view(torch.uint8))
               for a, b in zip(shard.segments, saved))


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


@pytest.mark.parametrize("nbytes", [0, 16, 1024, 32768 - 16, 32768, 32768 + 16, 5 * 32768 + 4096,
                                    64 * 4 * 32768, 3 * 64 * 4 * 32768 + 7 * 32768 + 48])
def test_copy_ceiling_copies_exactly(nbytes):
    # the bench's reference copy: whole tiles, a ragged last tile, several XCD rounds; the bytes
    # around the destination range stay as they were
    g = torch.Generator(device=DEV)
    g.manual_seed(nbytes + 1)
    src = torch.randint(0, 256, (nbytes + 64,), dtype=torch.uint8, device=DEV, generator=g)
    dst = torch.full((nbytes + 128,), 0xA5, dtype=torch.uint8, device=DEV)
    ff.ff_copy_ceiling(dst[64:], src, nbytes)
    torch.cuda.synchronize()
    assert torch.equal(dst[64:64 + nbytes], src[:nbytes])
    assert bool((dst[:64] == 0xA5).all()) and bool((dst[64 + nbytes:] == 0xA5).all())


@pytest.mark.parametrize("chunk,chained", [(1024, False), (1 << 16, False), (1 << 20, True), (4096, True)])
def test_mix_ceiling_moves_exactly_the_steps_bytes(chunk, chained):
    """The bench's ceiling for the optimizer steps' traffic: same tiles, loads and stores, no
    arithmetic, no CRC.  It is checked byte for byte: snapshot ranges of every group hold the
    gradient's bits (as the new 16-bit weights) and master, m, v unchanged; the tensors likewise;
    RAW ranges and the zero tail of the buffer are not touched."""
    numels = [1, 3, 255, 256, 257, 1000, 4095, 4096, 4097, 8191, 8192, 8193, 70001, 12289, 5, 77]
    shard = wl.param_shard("mix", numels, chunk, 9, DEV, with_grads=True)
    g = torch.Generator(device=DEV)
    g.manual_seed(2)
    raw = torch.randn(3001, device=DEV, generator=g)
    tensors = list(shard.segments)
    kinds, pids = [], []
    for pid in range(len(shard.params)):
        kinds += [ff.FF_KIND_W16, ff.FF_KIND_MASTER, ff.FF_KIND_M, ff.FF_KIND_V]
        pids += [pid] * 4
    tensors.insert(8, raw)
    kinds.insert(8, ff.FF_KIND_RAW)
    pids.insert(8, 0)
    plan = ff.ff_snapshot_plan(tensors, chunk, kinds=kinds, param_ids=pids)
    chunks, crcs, _, _ = ff.alloc_outputs(plan, DEV)
    grads = [p.grad for p in shard.params]
    before = [t.clone() for t in tensors]
    prev = None
    if chained:
        prev, prev_crcs, _, _ = ff.alloc_outputs(plan, DEV)
        ff.ff_pack(plan, prev, prev_crcs)          # the state the chained pattern reads
        for p in shard.params:
            for t in (p.master, p.m, p.v):
                t.view(torch.int32).fill_(0x7FC00BAD)
    chunks.fill_(0xA5)
    crcs.fill_(0x5A5A5A5A)
    ff.ff_mix_ceiling(plan, grads, prev, chunks)
    torch.cuda.synchronize()
    assert bool((crcs == 0x5A5A5A5A).all())
    got = chunks.cpu().numpy()
    covered = np.zeros(got.size, dtype=bool)
    for i, (t, b4) in enumerate(zip(tensors, before)):
        lo, hi = plan.segment_range(i)
        if kinds[i] == ff.FF_KIND_RAW:
            assert torch.equal(t, b4)
            continue
        covered[lo:hi] = True
        if kinds[i] == ff.FF_KIND_W16:
            want = wl.to_numpy_bytes(grads[pids[i]])
            assert np.array_equal(wl.to_numpy_bytes(t), want), i        # in place: gradient bits
        else:
            want = wl.to_numpy_bytes(b4)
            if chained:   # master, m, v tensors are neither read nor written
                assert bool((t.view(torch.int32) == 0x7FC00BAD).all()), i
            else:
                assert np.array_equal(wl.to_numpy_bytes(t), want), i
        assert np.array_equal(got[lo:hi], want), i
    assert bool((got[~covered] == 0xA5).all())


def test_one_plan_on_two_streams_at_once(oracle):
    """A plan is immutable: calls on ONE plan may overlap in time as long as their outputs differ.
    Two streams pack the same shard into two buffers and verify them concurrently, several times
    over (once with a corrupted chunk each); every result equals the oracle's."""
    shard = wl.param_shard("s", [1300000, 70001, 333, 250000], 1 << 18, 41, DEV, tiny_recipe=True)
    plan = ff.plan_for_shard(shard)
    want_buf, want_crcs = oracle.pack(_host_segments(shard)[0], shard.chunk_bytes, threads=8)
    outs = [ff.alloc_outputs(plan, DEV) for _ in range(2)]
    streams = [torch.cuda.Stream() for _ in range(2)]
    for st in streams:
        st.wait_stream(torch.cuda.current_stream())
    dirty = []
    for rep in range(6):
        for k, ((chunks, crcs, bad, n_bad), st) in enumerate(zip(outs, streams)):
            if rep == 3:      # corrupt one chunk of each buffer between two rounds, in stream order
                with torch.cuda.stream(st):
                    chunks[(5 + k) * shard.chunk_bytes + 17] ^= 0x40
                ff.ff_restore(plan, chunks, crcs, bad, n_bad, flags=ff.FF_RESTORE_VERIFY_ONLY,
                              stream=st)
                with torch.cuda.stream(st):
                    dirty.append((bad.clone(), n_bad.clone()))
            ff.ff_pack(plan, chunks, crcs, stream=st)
            ff.ff_restore(plan, chunks, crcs, bad, n_bad, flags=ff.FF_RESTORE_VERIFY_ONLY, stream=st)
    for st in streams:
        st.synchronize()
    for k, (chunks, crcs, bad, n_bad) in enumerate(outs):
        assert np.array_equal(chunks.cpu().numpy(), want_buf)
        assert np.array_equal(_u32(crcs), want_crcs)
        assert int(n_bad.item()) == 0 and not bool(bad.any())
        dbad, dn = dirty[k]
        assert int(dn.item()) == 1 and torch.nonzero(dbad).flatten().tolist() == [5 + k]


def test_one_plan_two_host_threads(oracle):
    """The same from two host threads, each with its own stream and outputs, sharing the plan."""
    import threading
    shard = wl.param_shard("t", [900000, 12345, 400001], 1 << 17, 43, DEV, tiny_recipe=True)
    plan = ff.plan_for_shard(shard)
    want_buf, want_crcs = oracle.pack(_host_segments(shard)[0], shard.chunk_bytes, threads=8)
    outs = [ff.alloc_outputs(plan, DEV) for _ in range(2)]
    streams = [torch.cuda.Stream() for _ in range(2)]
    for st in streams:
        st.wait_stream(torch.cuda.current_stream())
    errors = []

    def worker(k):
        try:
            torch.cuda.set_device(0)
            chunks, crcs, bad, n_bad = outs[k]
            for _ in range(8):
                ff.ff_pack(plan, chunks, crcs, stream=streams[k])
                ff.ff_restore(plan, chunks, crcs, bad, n_bad, flags=ff.FF_RESTORE_VERIFY_ONLY,
                              stream=streams[k])
            streams[k].synchronize()
        except Exception as e:          # surfaced in the main thread below
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for chunks, crcs, bad, n_bad in outs:
        assert np.array_equal(chunks.cpu().numpy(), want_buf)
        assert np.array_equal(_u32(crcs), want_crcs) and int(n_bad.item()) == 0


def test_two_plans_on_two_streams_at_once(oracle):
    """Two shards packed and verified concurrently, each through its own plan, stream and
    buffers, several times over."""
    shards = [wl.param_shard("s%d" % k, [300000 + 7 * k, 70001, 333], 1 << 18, 40 + k, DEV,
                             tiny_recipe=True) for k in range(2)]
    plans = [ff.plan_for_shard(s) for s in shards]
    outs = [ff.alloc_outputs(p, DEV) for p in plans]
    streams = [torch.cuda.Stream() for _ in plans]
    for st in streams:
        st.wait_stream(torch.cuda.current_stream())
    for _ in range(5):
        for plan, (chunks, crcs, bad, n_bad), st in zip(plans, outs, streams):
            ff.ff_pack(plan, chunks, crcs, stream=st)
            ff.ff_restore(plan, chunks, crcs, bad, n_bad, flags=ff.FF_RESTORE_VERIFY_ONLY, stream=st)
    for st in streams:
        st.synchronize()
    for shard, (chunks, crcs, bad, n_bad) in zip(shards, outs):
        want_buf, want_crcs = oracle.pack(_host_segments(shard)[0], shard.chunk_bytes, threads=8)
        assert np.array_equal(chunks.cpu().numpy(), want_buf)
        assert np.array_equal(_u32(crcs), want_crcs) and int(n_bad.item()) == 0


# ---- fused AdamW step + snapshot -----------------------------------------------------------------

HP = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=1000)


def _adam_and_compare(oracle, numels, chunk, seed, hp=HP, extra_raw=None, half=torch.bfloat16,
                      loss_scale=1.0, flags=0):
    """Runs ff_adam_step_snapshot and the oracle's unfused definition (update, then pack) on the
    same inputs.  fp32 state: max relative error <= 1e-6 is the acceptance bound; the fixed
    operation order makes the two bit-identical, which is what is asserted.  16-bit weights: exact
    rounding of the GPU's own fp32 master.  Snapshot bytes and CRCs: bit-exact.
    half = torch.float16 runs the loss-scaled fp16 variant of both."""
    shard = wl.param_shard("a", numels, chunk, seed, DEV, with_grads=True, half=half,
                           loss_scale=loss_scale)
    tensors = list(shard.segments)
    kinds, pids = [], []
    for pid in range(len(shard.params)):
        kinds += [ff.FF_KIND_W16, ff.FF_KIND_MASTER, ff.FF_KIND_M, ff.FF_KIND_V]
        pids += [pid] * 4
    if extra_raw is not None:
        for pos, t in extra_raw:
            tensors.insert(pos, t)
            kinds.insert(pos, ff.FF_KIND_RAW)
            pids.insert(pos, 0)
    plan = ff.ff_snapshot_plan(tensors, chunk, flags=flags, kinds=kinds, param_ids=pids)
    assert plan.num_params == len(numels)
    # host copies for the oracle, taken before the in-place update
    host = [wl.to_numpy_bytes(t) for t in tensors]
    views = {id(t): h for t, h in zip(tensors, host)}
    params_np, grads_np = [], []
    for p in shard.params:
        params_np.append((views[id(p.w16)].view(np.uint16), views[id(p.master)].view(np.float32),
                          views[id(p.m)].view(np.float32), views[id(p.v)].view(np.float32)))
        grads_np.append(wl.to_numpy_bytes(p.grad).view(np.uint16))
    chunks, crcs, bad, n_bad = ff.alloc_outputs(plan, DEV)
    chunks.fill_(0xA5)
    crcs.fill_(-1)
    if half == torch.float16:
        inv = float(np.float32(1.0 / loss_scale))
        n_nonfinite = torch.full((1,), -1, dtype=torch.int64, device=DEV)
        ff.ff_adam_step_snapshot_f16(plan, [p.grad for p in shard.params], hp, inv, n_nonfinite,
                                     chunks, crcs)
        torch.cuda.synchronize()
        want_buf, want_crcs, want_bad = oracle.adam_snapshot_f16(params_np, grads_np, inv, host,
                                                                 chunk, hp, threads=8)
        assert int(n_nonfinite.item()) == want_bad == 0
    else:
        ff.ff_adam_step_snapshot(plan, [p.grad for p in shard.params], hp, chunks, crcs)
        torch.cuda.synchronize()
        want_buf, want_crcs = oracle.adam_snapshot(params_np, grads_np, host, chunk, hp, threads=8)
    for p, (w16, master, m, v) in zip(shard.params, params_np):
        for name, got_t, want in (("master", p.master, master), ("m", p.m, m), ("v", p.v, v)):
            got = got_t.cpu().numpy()
            rel = np.abs(got.astype(np.float64) - want) / np.maximum(np.abs(want), 1.1754944e-38)
            assert rel.max(initial=0.0) <= 1e-6, name
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), name
        # 16-bit weight: exact RNE of the GPU's own fp32 master
        got_w = wl.to_numpy_bytes(p.w16).view(np.uint16)
        assert np.array_equal(got_w, wl.to_numpy_bytes(p.master.to(half)).view(np.uint16))
        assert np.array_equal(got_w, w16)
    assert np.array_equal(chunks.cpu().numpy(), want_buf)
    assert np.array_equal(_u32(crcs), want_crcs)
    # fused == unfused: ff_pack of the in-place result gives the same snapshot
    chunks2, crcs2, _, _ = ff.alloc_outputs(plan, DEV)
    ff.ff_pack(plan, chunks2, crcs2)
    torch.cuda.synchronize()
    assert torch.equal(chunks, chunks2) and torch.equal(crcs, crcs2)
    return shard, plan


@pytest.mark.parametrize("chunk", [1024, 4096, 1 << 16, 1 << 20])
def test_fused_adam_small_ragged(oracle, chunk):
    # odd element counts put fp32 segments at stream offsets 2 mod 4, so elements straddle
    # chunk boundaries; counts below and above one 256-element row and several tiles
    numels = [1, 3, 255, 256, 257, 1000, 4097, 70001, 131072, 65536 + 255, 5, 77]
    _adam_and_compare(oracle, numels, chunk, seed=chunk)


def test_fused_adam_many_random_sizes(oracle):
    numels = [int(x) for x in np.random.default_rng(42).integers(1, 30000, size=60)]
    _adam_and_compare(oracle, numels, 8192, seed=42)


def test_fused_adam_more_groups_than_one_launch_carries(oracle):
    # the gradient pointers travel in kernel arguments, 384 groups per launch: 1000 groups take
    # three launches, the last one partly filled
    numels = [int(x) for x in np.random.default_rng(43).integers(1, 700, size=1000)]
    _adam_and_compare(oracle, numels, 4096, seed=43)


@pytest.mark.parametrize("step", [1, 2, 1000])
def test_fused_adam_steps_and_hparams(oracle, step):
    hp = dict(lr=1e-3, beta1=0.8, beta2=0.999, eps=1e-6, weight_decay=0.0, step=step)
    _adam_and_compare(oracle, [5000, 12345, 300], 4096, seed=step, hp=hp)


def test_fused_adam_with_raw_segments(oracle):
    g = torch.Generator(device=DEV)
    g.manual_seed(3)
    raw1 = torch.randn(3001, device=DEV, generator=g)
    raw2 = torch.randn(70000, device=DEV, generator=g).to(torch.bfloat16)
    raw3 = torch.randn(9, device=DEV, generator=g).to(torch.bfloat16)
    _adam_and_compare(oracle, [1000, 33333, 77], 4096, seed=9,
                      extra_raw=[(0, raw1), (5, raw2), (14, raw3)])


def test_fused_adam_special_values(oracle):
    # zeros, denormals, infinities and NaNs in the state flow through identically
    shard = wl.param_shard("a", [4096], 4096, 5, DEV, with_grads=True)
    p = shard.params[0]
    p.v[:8] = torch.tensor([0.0, 1e-45, 1e-40, 1e-38, float("inf"), 0.0, 1e-30, 4.0], device=DEV)
    p.m[:8] = torch.tensor([0.0, 1e-45, -1e-40, float("nan"), 1.0, float("inf"), -0.0, 1e-20], device=DEV)
    p.master[8:12] = torch.tensor([float("nan"), float("inf"), -float("inf"), 3.4e38], device=DEV)
    p.grad[12:16] = torch.tensor([0.0, -0.0, 1e-38, 65504.0], device=DEV).to(torch.bfloat16)
    host = [wl.to_numpy_bytes(t) for t in shard.segments]
    params_np = [(host[0].view(np.uint16), host[1].view(np.float32), host[2].view(np.float32),
                  host[3].view(np.float32))]
    grads_np = [wl.to_numpy_bytes(p.grad).view(np.uint16)]
    plan = ff.plan_for_shard(shard)
    chunks, crcs, _, _ = ff.alloc_outputs(plan, DEV)
    ff.ff_adam_step_snapshot(plan, [p.grad], HP, chunks, crcs)
    torch.cuda.synchronize()
    want_buf, want_crcs = oracle.adam_snapshot(params_np, grads_np, host, 4096, HP)
    # A NaN result is stored as the canonical quiet NaN by both sides, so state, snapshot and CRCs
    # are compared byte for byte like everything else.
    n_nan = 0
    for got_t, want, bits in ((p.w16, params_np[0][0], 16), (p.master, params_np[0][1], 32),
                              (p.m, params_np[0][2], 32), (p.v, params_np[0][3], 32)):
        got = wl.to_numpy_bytes(got_t).view(np.uint16 if bits == 16 else np.uint32)
        want = want.view(got.dtype)
        assert np.array_equal(got, want)
        emask, fmask = (0x7F80, 0x007F) if bits == 16 else (0x7F800000, 0x007FFFFF)
        nan = ((got & emask) == emask) & ((got & fmask) != 0)
        n_nan += int(nan.sum())
        assert bool((got[nan] == (0x7FC0 if bits == 16 else 0x7FC00000)).all())
    assert n_nan >= 3
    assert np.array_equal(chunks.cpu().numpy(), want_buf)
    assert np.array_equal(_u32(crcs), want_crcs)
    # and the snapshot is the packed image of the state the GPU left in place
    chunks2, crcs2, _, _ = ff.alloc_outputs(plan, DEV)
    ff.ff_pack(plan, chunks2, crcs2)
    torch.cuda.synchronize()
    assert torch.equal(chunks, chunks2) and torch.equal(crcs, crcs2)


def test_fused_adam_argument_errors():
    shard = wl.param_shard("a", [100], 1024, 5, DEV, with_grads=True)
    p = shard.params[0]
    plan = ff.plan_for_shard(shard)
    chunks, crcs, _, _ = ff.alloc_outputs(plan, DEV)
    with pytest.raises(ff.FFError) as e:
        ff.ff_adam_step_snapshot(plan, [p.grad], dict(HP, step=0), chunks, crcs)
    assert e.value.status == ff.FF_ERR_INVALID
    # a plan without complete groups has nothing to step
    raw = ff.ff_snapshot_plan([p.master, p.m], 1024)
    with pytest.raises(ff.FFError) as e:
        ff.ff_adam_step_snapshot(raw, [p.grad], HP, chunks, crcs)
    assert e.value.status == ff.FF_ERR_INVALID


def test_fused_adam_consecutive_steps_and_new_gradient_buffers(oracle):
    """Three steps on one plan: the same gradient buffers twice, then different buffers (the
    pointers travel with every call).  The oracle takes the same three steps."""
    numels = [3000, 70001, 255]
    shard = wl.param_shard("a", numels, 4096, 21, DEV, with_grads=True)
    plan = ff.plan_for_shard(shard)
    host = [wl.to_numpy_bytes(t) for t in shard.segments]
    params_np = [(host[4 * i].view(np.uint16), host[4 * i + 1].view(np.float32),
                  host[4 * i + 2].view(np.float32), host[4 * i + 3].view(np.float32))
                 for i in range(len(numels))]
    chunks, crcs, _, _ = ff.alloc_outputs(plan, DEV)
    g = torch.Generator(device=DEV)
    g.manual_seed(77)
    grads_a = [p.grad for p in shard.params]
    grads_b = [torch.randn(n, device=DEV, generator=g).mul_(1e-3).to(torch.bfloat16) for n in numels]
    for step, grads in ((1, grads_a), (2, grads_a), (3, grads_b)):
        hp = dict(HP, step=step)
        if step == 2:
            for t in grads_a:                       # new values in the same buffers
                t.copy_(torch.randn(t.numel(), device=DEV, generator=g).mul_(1e-3))
        ff.ff_adam_step_snapshot(plan, grads, hp, chunks, crcs)
        torch.cuda.synchronize()
        grads_np = [wl.to_numpy_bytes(t).view(np.uint16) for t in grads]
        want_buf, want_crcs = oracle.adam_snapshot(params_np, grads_np, host, 4096, hp)
        assert np.array_equal(chunks.cpu().numpy(), want_buf), step
        assert np.array_equal(_u32(crcs), want_crcs), step
        for t, h in zip(shard.segments, host):
            assert np.array_equal(wl.to_numpy_bytes(t), h), step

def test_hip_graph_replays_of_the_whole_step():
    """The device entry points only launch kernels (the gradient pointers of the fused step are
    kernel arguments), so a step can be captured into a HIP graph.  Every replay, with eager work
    between replays, must equal the eager result."""
    numels = [3000, 70001, 255, 40000]
    shard = wl.param_shard("a", numels, 1 << 16, 33, DEV, with_grads=True)
    plan = ff.plan_for_shard(shard)
    grads = [p.grad for p in shard.params]
    chunks, crcs, bad, n_bad = ff.alloc_outputs(plan, DEV)
    pk, pcrcs, _, _ = ff.alloc_outputs(plan, DEV)

    def step():
        ff.ff_adam_step_snapshot(plan, grads, HP, chunks, crcs)
        ff.ff_pack(plan, pk, pcrcs)
        ff.ff_restore(plan, chunks, crcs, bad, n_bad)

    step()                                           # warm-up: the first launch loads the kernels
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)
    for rep in range(3):
        start = [t.clone() for t in shard.segments]
        for t in grads:                              # eager work between the replays
            t.copy_(torch.randn(t.numel(), device=DEV, generator=gen).mul_(1e-3))
        for out in (chunks, pk):
            out.fill_(0xA5)
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in shard.segments] + [chunks.clone(), crcs.clone(), pk.clone(),
                                                     pcrcs.clone(), bad.clone(), n_bad.clone()]
        for t, s0 in zip(shard.segments, start):
            t.copy_(s0)
        for out in (chunks, pk):
            out.fill_(0xA5)
        step()
        torch.cuda.synchronize()
        want = list(shard.segments) + [chunks, crcs, pk, pcrcs, bad, n_bad]
        for a, b in zip(got, want):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), rep
        assert int(n_bad.item()) == 0 and torch.equal(chunks, pk) and torch.equal(crcs, pcrcs)


def test_hip_graph_replays_of_two_chained_steps():
    """Two chained steps, A -> B -> A, captured as one graph: every replay advances the state in
    the snapshots by two steps and must equal the same two steps taken eagerly."""
    numels = [3000, 70001, 255, 40000]
    shard = wl.param_shard("a", numels, 1 << 16, 35, DEV, with_grads=True)
    plan = ff.plan_for_shard(shard)
    grads = [p.grad for p in shard.params]
    a, crcs_a, bad, n_bad = ff.alloc_outputs(plan, DEV)
    b, crcs_b, _, _ = ff.alloc_outputs(plan, DEV)
    ff.ff_pack(plan, a, crcs_a)

    def two_steps():
        ff.ff_adam_step_chained(plan, grads, HP, a, b, crcs_b)
        ff.ff_adam_step_chained(plan, grads, HP, b, a, crcs_a)

    start = a.clone()
    two_steps()                                      # warm-up: the first launch loads the kernels
    torch.cuda.synchronize()
    a.copy_(start)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        two_steps()
    gen = torch.Generator(device=DEV)
    gen.manual_seed(6)
    for rep in range(3):
        start = a.clone()
        for t in grads:                              # eager work between the replays
            t.copy_(torch.randn(t.numel(), device=DEV, generator=gen).mul_(1e-3))
        b.fill_(0xA5)
        graph.replay()
        torch.cuda.synchronize()
        got = [x.clone() for x in (a, crcs_a, b, crcs_b)] + [p.w16.clone() for p in shard.params]
        a.copy_(start)
        b.fill_(0xA5)
        two_steps()
        torch.cuda.synchronize()
        want = [a, crcs_a, b, crcs_b] + [p.w16 for p in shard.params]
        for x, y in zip(got, want):
            assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), rep
        assert not torch.equal(a, start)
        ff.ff_restore(plan, a, crcs_a, bad, n_bad, ff.FF_RESTORE_VERIFY_ONLY)
        torch.cuda.synchronize()
        assert int(n_bad.item()) == 0


@pytest.mark.parametrize("seed", list(range(10)))
def test_fused_adam_random_cases(oracle, seed):
    """Seeded random shapes: group sizes from one element to a few tiles, any chunk size, RAW
    tensors of both widths sprinkled between the groups, either 16-bit format."""
    rng = np.random.default_rng(1000 + seed)
    n_groups = int(rng.integers(1, 10))
    numels = [int(rng.choice([rng.integers(1, 600), rng.integers(600, 9000), rng.integers(9000, 60000)]))
              for _ in range(n_groups)]
    chunk = int(rng.choice([1024, 2048, 16384, 65536, 1 << 18]))
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    extra = []
    for _ in range(int(rng.integers(0, 4))):
        n = int(rng.integers(1, 5000))
        dt = torch.float32 if rng.random() < 0.5 else torch.bfloat16
        pos = int(rng.integers(0, 4 * n_groups + 1)) // 4 * 4        # between two groups
        extra.append((pos, torch.randn(n, device=DEV, generator=g).to(dt)))
    extra.sort(key=lambda e: -e[0])                                  # insert from the back
    half = torch.float16 if seed % 2 else torch.bfloat16
    hp = dict(lr=float(rng.choice([1e-4, 3e-3])), beta1=0.9, beta2=float(rng.choice([0.95, 0.999])),
              eps=1e-8, weight_decay=float(rng.choice([0.0, 0.1])), step=int(rng.integers(1, 2000)))
    _adam_and_compare(oracle, numels, chunk, seed=2000 + seed, hp=hp, extra_raw=extra or None,
                      half=half, loss_scale=1024.0 if seed % 2 else 1.0)
    if seed < 6:  # the same shapes with the state kept in the snapshots
        _chained_and_compare(oracle, numels, chunk, seed=2500 + seed, steps=2,
                             extra_raw=extra or None, half=half,
                             loss_scale=1024.0 if seed % 2 else 1.0)


@pytest.mark.parametrize("seed", list(range(8)))
def test_pack_restore_random_layouts_and_tiles(oracle, seed):
    rng = np.random.default_rng(3000 + seed)
    mu = float(rng.uniform(4.0, 10.0))
    lay = wl.fragmented_layout(seed=3000 + seed, n_tensors=int(rng.integers(20, 800)), mu=mu,
                               sigma=float(rng.uniform(0.5, 2.5)), max_numel=1 << 17)
    chunk = int(rng.choice([1024, 8192, 1 << 15, 1 << 16, 1 << 19]))
    tile_log2 = int(rng.choice([0, 0, 10, 12, 14, 16]))
    shard = wl.fragmented_shard(lay, chunk, seed=seed, device=DEV)
    state = _pack_and_compare(shard, oracle, tile_log2)
    _restore_and_compare(shard, *state[:6])


def test_fused_adam_with_large_raw_segments(oracle):
    # RAW segments long enough that the RAW kernel's XCD-aware order permutes complete rounds of
    # tiles (8 MiB each), between and around parameter groups
    g = torch.Generator(device=DEV)
    g.manual_seed(31)
    raw1 = torch.randn(5 * (1 << 20) + 3, device=DEV, generator=g)                     # 20 MiB + 12 B
    raw2 = torch.randn(3 * (1 << 20) + 1, device=DEV, generator=g).to(torch.bfloat16)  # 6 MiB + 2 B
    raw3 = torch.randn(2500001, device=DEV, generator=g)                               # 9.5 MiB
    _adam_and_compare(oracle, [50000, 300001], 1 << 20, seed=12,
                      extra_raw=[(0, raw1), (5, raw2), (10, raw3)])


# Tuning flags of a plan change the order and the cache policy of the accesses, never the result.
_TUNING = [ff.FF_PLAN_XCD_ORDER(1), ff.FF_PLAN_XCD_ORDER(2), ff.FF_PLAN_XCD_ORDER(3),
           ff.FF_PLAN_XCD_ORDER(31), ff.FF_PLAN_CACHE_HINT(0),
           ff.FF_PLAN_CACHE_HINT(1) | ff.FF_PLAN_XCD_ORDER(1), ff.FF_PLAN_CACHE_HINT(2)]


@pytest.mark.parametrize("flags", _TUNING)
def test_plan_tuning_flags_pack_restore(oracle, flags):
    # 6 MiB in 32 KiB tiles: runs of 1, 2 and 4 workgroups per XCD permute several complete rounds
    lay = wl.fragmented_layout(seed=77, n_tensors=120, mu=9.5, sigma=1.5, max_numel=1 << 18)
    shard = wl.fragmented_shard(lay, 1 << 18, seed=flags, device=DEV)
    assert sum(n for _, n in shard.spans) > 3 << 20
    state = _pack_and_compare(shard, oracle, flags=flags)
    _restore_and_compare(shard, *state[:6])
    plan, chunks, crcs, bad, n_bad = state[:5]
    ff.ff_restore(plan, chunks, crcs, bad, n_bad, ff.FF_RESTORE_VERIFY_ONLY)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0


@pytest.mark.parametrize("flags", _TUNING)
def test_plan_tuning_flags_fused_step(oracle, flags):
    # 40 and more tiles of 8192 elements: complete rounds for runs of 1, 2 and 4
    _adam_and_compare(oracle, [200000, 77777, 5, 131072], 1 << 16, seed=flags, flags=flags)


# ---- the step that reads its state from the previous snapshot ------------------------------------

def _chained_and_compare(oracle, numels, chunk, seed, steps=3, half=torch.bfloat16, loss_scale=1.0,
                         extra_raw=None, flags=0):
    """ff_adam_step_chained over `steps` steps that alternate between two snapshot buffers, against
    the oracle's definition step by step: snapshot bytes and CRCs bit-exact (which holds the fp32
    state to the bit, inside the 1e-6 bound), working weights exact, MASTER/M/V tensors untouched.
    Then one more step both ways: chained, and in place on tensors restored from the snapshot."""
    shard = wl.param_shard("a", numels, chunk, seed, DEV, with_grads=True, half=half,
                           loss_scale=loss_scale)
    tensors = list(shard.segments)
    kinds, pids = [], []
    for pid in range(len(shard.params)):
        kinds += [ff.FF_KIND_W16, ff.FF_KIND_MASTER, ff.FF_KIND_M, ff.FF_KIND_V]
        pids += [pid] * 4
    for pos, t in (extra_raw or []):
        tensors.insert(pos, t)
        kinds.insert(pos, ff.FF_KIND_RAW)
        pids.insert(pos, 0)
    plan = ff.ff_snapshot_plan(tensors, chunk, flags=flags, kinds=kinds, param_ids=pids)
    host = [wl.to_numpy_bytes(t) for t in tensors]
    views = {id(t): h for t, h in zip(tensors, host)}
    params_np, grads_np = [], []
    for p in shard.params:
        params_np.append((views[id(p.w16)].view(np.uint16), views[id(p.master)].view(np.float32),
                          views[id(p.m)].view(np.float32), views[id(p.v)].view(np.float32)))
        grads_np.append(wl.to_numpy_bytes(p.grad).view(np.uint16))
    grads = [p.grad for p in shard.params]
    bufs = [ff.alloc_outputs(plan, DEV)[:2] for _ in range(2)]
    ff.ff_pack(plan, *bufs[0])                     # snapshot 0: the initial state
    torch.cuda.synchronize()
    prev_np, prev_crcs = oracle.pack(host, chunk, threads=8)
    assert np.array_equal(bufs[0][0].cpu().numpy(), prev_np)
    # from here on the optimizer state lives in the snapshots: the tensors hold poison
    for p in shard.params:
        for t in (p.master, p.m, p.v):
            t.view(torch.int32).fill_(0x7FC00BAD)
    f16 = half == torch.float16
    inv = float(np.float32(1.0 / loss_scale)) if f16 else 1.0
    n_nonfinite = torch.full((1,), -1, dtype=torch.int64, device=DEV) if f16 else None
    for k in range(steps):
        hp = dict(HP, step=HP["step"] + k)
        src, (dst, dst_crcs) = bufs[k % 2][0], bufs[(k + 1) % 2]
        dst.fill_(0xA5)
        dst_crcs.fill_(-1)
        ff.ff_adam_step_chained(plan, grads, hp, src, dst, dst_crcs, inv, n_nonfinite)
        torch.cuda.synchronize()
        want_buf, want_crcs, want_bad = oracle.adam_snapshot_chained(
            prev_np, params_np, grads_np, host, chunk, hp, inv_scale=inv if f16 else None, threads=8)
        assert np.array_equal(dst.cpu().numpy(), want_buf), k
        assert np.array_equal(_u32(dst_crcs), want_crcs), k
        if f16:
            assert int(n_nonfinite.item()) == want_bad == 0
        for p, (w16, _, _, _) in zip(shard.params, params_np):
            assert np.array_equal(wl.to_numpy_bytes(p.w16).view(np.uint16), w16)
            for t in (p.master, p.m, p.v):
                assert bool((t.view(torch.int32) == 0x7FC00BAD).all())
        prev_np = want_buf
    # the chain equals the in-place step: load the last snapshot into the tensors and step both ways
    last, (other, other_crcs) = bufs[steps % 2], bufs[(steps + 1) % 2]
    _, _, bad, n_bad = ff.alloc_outputs(plan, DEV)
    hp = dict(HP, step=HP["step"] + steps)
    ff.ff_adam_step_chained(plan, grads, hp, last[0], other, other_crcs, inv, n_nonfinite)
    torch.cuda.synchronize()
    chained_buf, chained_crcs = other.cpu().numpy().copy(), _u32(other_crcs).copy()
    ff.ff_restore(plan, last[0], last[1], bad, n_bad)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0
    if f16:
        ff.ff_adam_step_snapshot_f16(plan, grads, hp, inv, n_nonfinite, other, other_crcs)
    else:
        ff.ff_adam_step_snapshot(plan, grads, hp, other, other_crcs)
    torch.cuda.synchronize()
    assert np.array_equal(other.cpu().numpy(), chained_buf)
    assert np.array_equal(_u32(other_crcs), chained_crcs)


@pytest.mark.parametrize("chunk", [1024, 4096, 1 << 16, 1 << 20])
def test_chained_step_small_ragged(oracle, chunk):
    numels = [1, 3, 255, 256, 257, 1000, 4097, 70001, 131072, 65536 + 255, 5, 77]
    _chained_and_compare(oracle, numels, chunk, seed=chunk + 2)


def test_chained_step_with_raw_segments_and_tuning_flags(oracle):
    g = torch.Generator(device=DEV)
    g.manual_seed(5)
    raw1 = torch.randn(3001, device=DEV, generator=g)
    raw2 = torch.randn(70001, device=DEV, generator=g).to(torch.bfloat16)  # fp32 streams at 2 mod 4
    raw3 = torch.randn(9, device=DEV, generator=g).to(torch.bfloat16)
    _chained_and_compare(oracle, [1000, 33333, 77, 200000], 4096, seed=19,
                         extra_raw=[(0, raw1), (5, raw2), (14, raw3)],
                         flags=ff.FF_PLAN_XCD_ORDER(1))


@pytest.mark.parametrize("loss_scale", [1.0, 4096.0])
def test_chained_step_f16(oracle, loss_scale):
    _chained_and_compare(oracle, [5000, 12345, 300, 3], 4096, seed=23, half=torch.float16,
                         loss_scale=loss_scale)


def test_chained_step_argument_errors():
    shard = wl.param_shard("a", [5000], 4096, 5, DEV, with_grads=True)
    plan = ff.plan_for_shard(shard)
    a, crcs, _, _ = ff.alloc_outputs(plan, DEV)
    both = torch.zeros(2 * a.numel() + 64, dtype=torch.uint8, device=DEV)
    grads = [shard.params[0].grad]
    n_nonfinite = torch.zeros(1, dtype=torch.int64, device=DEV)
    n = a.numel()
    cases = [
        lambda: ff.ff_adam_step_chained(plan, grads, HP, a, a, crcs),                        # the same buffer
        lambda: ff.ff_adam_step_chained(plan, grads, HP, both[16:16 + n], both[:n], crcs),   # overlapping
        lambda: ff.ff_adam_step_chained(plan, grads, HP, both[n - 16:2 * n - 16], both[:n], crcs),
        lambda: ff.ff_adam_step_chained(plan, grads, HP, both[n + 8:2 * n + 8], both[:n], crcs),  # misaligned
        lambda: ff.ff_adam_step_chained(plan, grads, HP, both[n:2 * n], both[:n], crcs, 0.5),     # bf16 plan
        lambda: ff.ff_adam_step_chained(plan, grads, HP, both[n:2 * n], both[:n], crcs, 1.0, n_nonfinite),
        lambda: ff.ff_adam_step_chained(plan, grads, dict(HP, step=0), both[n:2 * n], both[:n], crcs),
    ]
    for case in cases:
        with pytest.raises(ff.FFError) as e:
            case()
        assert e.value.status == ff.FF_ERR_INVALID
    ff.ff_adam_step_chained(plan, grads, HP, both[n:2 * n], both[:n], crcs)   # adjacent buffers are fine
    torch.cuda.synchronize()


# ---- fp16 variant of the fused step ---------------------------------------------------------------

@pytest.mark.parametrize("chunk,loss_scale", [(1024, 1.0), (4096, 1024.0), (1 << 16, 65536.0),
                                              (1 << 20, 128.0)])
def test_fused_adam_f16_small_ragged(oracle, chunk, loss_scale):
    numels = [1, 3, 255, 256, 257, 1000, 4097, 70001, 131072, 65536 + 255, 5, 77]
    _adam_and_compare(oracle, numels, chunk, seed=chunk + 1, half=torch.float16,
                      loss_scale=loss_scale)


@pytest.mark.parametrize("step", [1, 2, 1000])
def test_fused_adam_f16_steps_and_hparams(oracle, step):
    hp = dict(lr=1e-3, beta1=0.8, beta2=0.999, eps=1e-6, weight_decay=0.0, step=step)
    _adam_and_compare(oracle, [5000, 12345, 300], 4096, seed=step, hp=hp, half=torch.float16,
                      loss_scale=4096.0)


def test_fused_adam_f16_with_raw_segments(oracle):
    g = torch.Generator(device=DEV)
    g.manual_seed(3)
    raw1 = torch.randn(3001, device=DEV, generator=g)
    raw2 = torch.randn(70000, device=DEV, generator=g).to(torch.float16)
    _adam_and_compare(oracle, [1000, 33333, 77], 4096, seed=9, extra_raw=[(0, raw1), (5, raw2)],
                      half=torch.float16, loss_scale=512.0)


def test_fused_adam_f16_nonfinite_gradients_and_weight_overflow(oracle):
    n = 5000
    shard = wl.param_shard("a", [n, 300], 4096, 6, DEV, with_grads=True, half=torch.float16,
                           loss_scale=1024.0)
    p = shard.params[0]
    inf = float("inf")
    p.grad[:6] = torch.tensor([inf, -inf, float("nan"), 65504.0, -65504.0, 6e-8], device=DEV).to(torch.float16)
    p.grad[4097] = inf                                   # second tile row range, another chunk
    shard.params[1].grad[299] = float("nan")
    # masters beyond the fp16 range round to infinity
    p.master[10:16] = torch.tensor([65519.0, 65530.0, -70000.0, 1e-7, -3e-8, 3.4e38], device=DEV)
    host = [wl.to_numpy_bytes(t) for t in shard.segments]
    params_np = [(host[4 * i].view(np.uint16), host[4 * i + 1].view(np.float32),
                  host[4 * i + 2].view(np.float32), host[4 * i + 3].view(np.float32))
                 for i in range(2)]
    grads_np = [wl.to_numpy_bytes(q.grad).view(np.uint16) for q in shard.params]
    plan = ff.plan_for_shard(shard)
    chunks, crcs, _, _ = ff.alloc_outputs(plan, DEV)
    n_nonfinite = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    inv = float(np.float32(1.0 / 1024.0))
    ff.ff_adam_step_snapshot_f16(plan, [q.grad for q in shard.params], HP, inv, n_nonfinite,
                                 chunks, crcs)
    torch.cuda.synchronize()
    want_buf, want_crcs, want_bad = oracle.adam_snapshot_f16(params_np, grads_np, inv, host, 4096, HP)
    assert want_bad == 5 and int(n_nonfinite.item()) == 5
    # NaN results are stored in the canonical form on both sides: everything bit for bit
    n_nan = 0
    for q, (w16, master, m, v) in zip(shard.params, params_np):
        for got_t, want in ((q.master, master), (q.m, m), (q.v, v)):
            got = got_t.cpu().numpy()
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
            assert bool((got.view(np.uint32)[np.isnan(got)] == 0x7FC00000).all())
            n_nan += int(np.isnan(got).sum())
        got_w = wl.to_numpy_bytes(q.w16).view(np.uint16)
        assert np.array_equal(got_w, w16)
        assert bool((got_w[np.isnan(got_w.view(np.float16))] == 0x7E00).all())
    assert n_nan >= 3
    assert np.array_equal(chunks.cpu().numpy(), want_buf)
    assert np.array_equal(_u32(crcs), want_crcs)
    w = wl.to_numpy_bytes(p.w16).view(np.uint16)
    assert w[11] == 0x7C00 and w[12] == 0xFC00 and w[15] == 0x7C00     # overflow to infinity
    assert w[10] == 0x7BFF                                             # 65519 * decay stays finite
    # n_nonfinite may be NULL; the snapshot equals ff_pack of the state left in place
    chunks2, crcs2, _, _ = ff.alloc_outputs(plan, DEV)
    ff.ff_pack(plan, chunks2, crcs2)
    torch.cuda.synchronize()
    assert torch.equal(chunks, chunks2) and torch.equal(crcs, crcs2)
    ff.ff_adam_step_snapshot_f16(plan, [q.grad for q in shard.params], HP, inv, None, chunks, crcs)
    torch.cuda.synchronize()


def test_fused_adam_format_mismatch_is_rejected():
    bf = wl.param_shard("b", [1000], 4096, 1, DEV, with_grads=True)
    fh = wl.param_shard("h", [1000], 4096, 1, DEV, with_grads=True, half=torch.float16)
    for shard, wrong in ((bf, "f16"), (fh, "bf16")):
        plan = ff.plan_for_shard(shard)
        chunks, crcs, _, _ = ff.alloc_outputs(plan, DEV)
        grads = [q.grad for q in shard.params]
        with pytest.raises(ff.FFError) as e:
            if wrong == "f16":
                ff.ff_adam_step_snapshot_f16(plan, grads, HP, 1.0, None, chunks, crcs)
            else:
                ff.ff_adam_step_snapshot(plan, grads, HP, chunks, crcs)
        assert e.value.status == ff.FF_ERR_INVALID
    # a plan that mixes the two 16-bit formats has no valid fused step; it still packs
    mixed = list(bf.segments) + list(fh.segments)
    kinds = [ff.FF_KIND_W16, ff.FF_KIND_MASTER, ff.FF_KIND_M, ff.FF_KIND_V] * 2
    plan = ff.ff_snapshot_plan(mixed, 4096, kinds=kinds, param_ids=[0] * 4 + [1] * 4)
    assert plan.num_params == 0
    chunks, crcs, _, _ = ff.alloc_outputs(plan, DEV)
    ff.ff_pack(plan, chunks, crcs)
    torch.cuda.synchronize()

# ---- selective restore ------------------------------------------------------------------------------

def _segments_as_stream(shard):
    return np.concatenate(_host_segments(shard)[0])


@pytest.mark.parametrize("chunk,tile_log2", [(1024, 0), (1 << 14, 12), (1 << 16, 0), (1 << 20, 0)])
def test_restore_chunks_matches_oracle(oracle, chunk, tile_log2):
    numels = [int(x) for x in np.random.default_rng(chunk + 1).integers(1, 60000, size=30)]
    shard = wl.param_shard("sel", numels, chunk, 31, DEV, tiny_recipe=True)
    plan, chunks, crcs, bad, n_bad, want_buf, want_crcs = _pack_and_compare(shard, oracle, tile_log2)
    n = plan.num_chunks
    rng = np.random.default_rng(7)
    ids = sorted({int(x) for x in rng.integers(0, n, size=max(2, n // 3))} | {0, n - 1})
    dirty = chunks.clone()
    flipped = ids[len(ids) // 2]
    dirty[flipped * chunk + 5] ^= 0x40                       # one listed chunk is corrupt
    other = next(j for j in range(n) if j not in ids)
    dirty[other * chunk + 9] ^= 0x01                         # an unlisted one too: must go unnoticed
    for flags, skip in ((0, False), (ff.FF_RESTORE_SKIP_BAD, True)):
        _poison_segments(shard)
        bad.fill_(7)
        n_bad.fill_(99)
        ff.ff_restore_chunks(plan, dirty, crcs, ids, bad, n_bad, flags=flags)
        torch.cuda.synchronize()
        # the oracle on host copies poisoned the same way
        host = [np.full(h.size, 0xA5, dtype=np.uint8) for h in _host_segments(shard)[0]]
        want_bad = np.full(n, 7, dtype=np.uint32)
        want_n = oracle.restore_chunks(host, chunk, dirty.cpu().numpy(), want_crcs, ids, want_bad,
                                       skip_bad=skip)
        assert want_n == 1
        assert int(n_bad.item()) == want_n
        assert np.array_equal(_u32(bad), want_bad)
        assert np.array_equal(_segments_as_stream(shard), np.concatenate(host))
    # an empty list only clears n_bad
    n_bad.fill_(5)
    ff.ff_restore_chunks(plan, dirty, crcs, [], bad, n_bad)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0
    L = ff.lib()
    import ctypes
    two = (ctypes.c_uint64 * 2)(3, 3)
    assert L.ff_restore_chunks(plan.handle, dirty.data_ptr(), crcs.data_ptr(), two, 2,
                               bad.data_ptr(), n_bad.data_ptr(), 0, None) == ff.FF_ERR_INVALID
    two = (ctypes.c_uint64 * 2)(0, n)
    assert L.ff_restore_chunks(plan.handle, dirty.data_ptr(), crcs.data_ptr(), two, 2,
                               bad.data_ptr(), n_bad.data_ptr(), 0, None) == ff.FF_ERR_INVALID


@pytest.mark.parametrize("flags", [0, ff.FF_RESTORE_SKIP_BAD, ff.FF_RESTORE_VERIFY_ONLY])
def test_restore_chunks_long_list(oracle, flags):
    """A list longer than one launch carries in its arguments (several launches per call): 700
    of 1000 chunks, some of them corrupt, against the oracle."""
    chunk = 1024
    numels = [int(x) for x in np.random.default_rng(77).integers(100, 30000, size=18)]
    shard = wl.param_shard("long", numels, chunk, 33, DEV, tiny_recipe=True)
    plan, chunks, crcs, bad, n_bad, want_buf, want_crcs = _pack_and_compare(shard, oracle)
    n = plan.num_chunks
    assert n > 900
    rng = np.random.default_rng(8)
    ids = sorted({int(x) for x in rng.choice(n, size=700, replace=False)})
    dirty = chunks.clone()
    flipped = [ids[3], ids[260], ids[511], ids[699]]          # first, middle and last launch
    for j in flipped:
        dirty[j * chunk + (j % 1000)] ^= 0x08
    _poison_segments(shard)
    bad.fill_(7)
    n_bad.fill_(99)
    ff.ff_restore_chunks(plan, dirty, crcs, ids, bad, n_bad, flags=flags)
    torch.cuda.synchronize()
    host = [np.full(h.size, 0xA5, dtype=np.uint8) for h in _host_segments(shard)[0]]
    want_bad = np.full(n, 7, dtype=np.uint32)
    if flags == ff.FF_RESTORE_VERIFY_ONLY:
        vb, _ = oracle.verify(dirty.cpu().numpy(), want_crcs, chunk)
        want_bad[ids] = vb[ids]
        want_n = int(vb[ids].sum())
    else:
        want_n = oracle.restore_chunks(host, chunk, dirty.cpu().numpy(), want_crcs, ids, want_bad,
                                       skip_bad=flags == ff.FF_RESTORE_SKIP_BAD)
    assert want_n == len(flipped) == int(n_bad.item())
    assert np.array_equal(_u32(bad), want_bad)
    assert np.array_equal(_segments_as_stream(shard), np.concatenate(host))


def test_swapped_chunks_are_both_flagged(oracle):
    """Chunk reorder on the way to the receiver: two chunks of the buffer change places while the
    CRC array keeps its order.  Exactly those two are flagged (their contents differ), by the
    oracle and by ff_restore alike; swapping the CRCs along makes the buffer verify again but
    it is then a different snapshot, which the byte comparison shows."""
    numels = [int(x) for x in np.random.default_rng(6).integers(1000, 90000, size=30)]
    shard = wl.param_shard("swap", numels, 1 << 16, 6, DEV, tiny_recipe=True)
    plan, chunks, crcs, bad, n_bad, want_buf, want_crcs = _pack_and_compare(shard, oracle)
    C, n = shard.chunk_bytes, plan.num_chunks
    a, b = 2, n - 3
    assert want_crcs[a] != want_crcs[b]
    moved = chunks.clone()
    moved[a * C:(a + 1) * C] = chunks[b * C:(b + 1) * C]
    moved[b * C:(b + 1) * C] = chunks[a * C:(a + 1) * C]
    for flags in (0, ff.FF_RESTORE_VERIFY_ONLY, ff.FF_RESTORE_SKIP_BAD):
        _poison_segments(shard)
        ff.ff_restore(plan, moved, crcs, bad, n_bad, flags=flags)
        torch.cuda.synchronize()
        want_bad, want_n = oracle.verify(moved.cpu().numpy(), want_crcs, C)
        assert want_n == 2 and list(np.nonzero(want_bad)[0]) == [a, b]
        assert int(n_bad.item()) == 2 and np.array_equal(_u32(bad), want_bad)
    # the skip-bad pass left the two chunks' tensor ranges untouched and loaded the rest
    got = _segments_as_stream(shard)
    for j in range(n):
        lo, hi = j * C, min((j + 1) * C, got.size)
        if j in (a, b):
            assert bool((got[lo:hi] == 0xA5).all())
        else:
            assert np.array_equal(got[lo:hi], want_buf[lo:hi])
    crcs_moved = crcs.clone()
    crcs_moved[a], crcs_moved[b] = crcs[b], crcs[a]
    ff.ff_restore(plan, moved, crcs_moved, bad, n_bad, flags=ff.FF_RESTORE_VERIFY_ONLY)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0


def test_restore_checked_refuses_another_layout(oracle):
    """A buffer packed for one layout offered to a plan with another one: ff_restore_checked
    returns FF_ERR_LAYOUT and writes nothing -- no tensor byte, no bad[], no n_bad; with the
    matching id it is ff_restore."""
    numels = [30000, 70001, 4096]
    C = 1 << 15
    sender = wl.param_shard("snd", numels, C, 3, DEV, tiny_recipe=True)
    plan_s, chunks, crcs, bad, n_bad, want_buf, want_crcs = _pack_and_compare(sender, oracle)
    # receivers: same sizes in another order; one element more; another chunk size
    others = [wl.param_shard("r1", [70001, 30000, 4096], C, 4, DEV, tiny_recipe=True),
              wl.param_shard("r2", [30000, 70001, 4097], C, 4, DEV, tiny_recipe=True),
              wl.param_shard("r3", numels, 2 * C, 4, DEV, tiny_recipe=True)]
    for recv in others:
        plan_r = ff.plan_for_shard(recv)
        assert plan_r.layout_id != plan_s.layout_id
        _poison_segments(recv)
        n_r = plan_r.num_chunks
        bad_r = torch.full((max(n_r, plan_s.num_chunks),), 7, dtype=torch.int32, device=DEV)
        n_bad.fill_(99)
        big = torch.zeros(max(plan_r.buffer_bytes, plan_s.buffer_bytes), dtype=torch.uint8, device=DEV)
        big[:plan_s.buffer_bytes] = chunks
        crcs_r = torch.zeros(max(n_r, plan_s.num_chunks), dtype=torch.int32, device=DEV)
        crcs_r[:plan_s.num_chunks] = crcs
        with pytest.raises(ff.FFError) as e:
            ff.ff_restore_checked(plan_r, plan_s.layout_id, big, crcs_r, bad_r, n_bad)
        assert e.value.status == ff.FF_ERR_LAYOUT
        torch.cuda.synchronize()
        assert all(bool((t.view(torch.uint8) == 0xA5).all()) for t in recv.segments)
        assert bool((bad_r == 7).all()) and int(n_bad.item()) == 99
    # a receiver with the sender's layout (fresh tensors, other addresses) loads the state
    recv = wl.param_shard("r0", numels, C, 9, DEV, tiny_recipe=True)
    plan_r = ff.plan_for_shard(recv)
    assert plan_r.layout_id == plan_s.layout_id
    _poison_segments(recv)
    ff.ff_restore_checked(plan_r, plan_s.layout_id, chunks, crcs, bad, n_bad)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0
    got = _segments_as_stream(recv)
    assert np.array_equal(got, want_buf[:got.size])


def test_full_restore_skip_bad_on_ragged_layout(oracle):
    lay = wl.fragmented_layout(seed=4, n_tensors=1500, mu=6.0, sigma=2.0, max_numel=1 << 16)
    shard = wl.fragmented_shard(lay, 1 << 14, seed=4, device=DEV)
    plan, chunks, crcs, bad, n_bad, want_buf, want_crcs = _pack_and_compare(shard, oracle)
    n, C = plan.num_chunks, shard.chunk_bytes
    hits = wl.corrupt_chunks(n, C, seed=4, fraction=0.05)
    dirty = chunks.clone()
    for c, off, bit in hits:
        dirty[c * C + off] ^= (1 << bit)
    before = shard.arena.clone()
    _poison_segments(shard)
    poisoned = shard.arena.cpu().numpy().copy()
    ff.ff_restore(plan, dirty, crcs, bad, n_bad, flags=ff.FF_RESTORE_SKIP_BAD)
    torch.cuda.synchronize()
    arena = poisoned.copy()
    host = [arena[o:o + nb] for o, nb in shard.spans]
    want_bad = np.zeros(n, dtype=np.uint32)
    want_n = oracle.restore_chunks(host, C, dirty.cpu().numpy(), want_crcs, np.arange(n), want_bad,
                                   skip_bad=True)
    assert want_n == len(hits) and int(n_bad.item()) == want_n
    assert np.array_equal(_u32(bad), want_bad)
    assert np.array_equal(shard.arena.cpu().numpy(), arena)   # gaps and skipped ranges untouched


# ---- snapshot into pinned host memory ----------------------------------------------------------------

@pytest.mark.parametrize("slice_chunks", [1, 5, 1000])
def test_pack_to_host_equals_pack(oracle, slice_chunks):
    numels = [int(x) for x in np.random.default_rng(3).integers(1, 90000, size=40)]
    shard = wl.param_shard("h", numels, 1 << 16, 17, DEV, tiny_recipe=True)
    plan = ff.plan_for_shard(shard)
    chunks, crcs, bad, n_bad = ff.alloc_outputs(plan, DEV)
    chunks.fill_(0xA5)
    h_chunks = torch.empty(plan.buffer_bytes, dtype=torch.uint8, pin_memory=True).fill_(0x5A)
    h_crcs = torch.empty(plan.num_chunks, dtype=torch.int32, pin_memory=True).fill_(-1)
    s_pack, s_copy = torch.cuda.Stream(), torch.cuda.Stream()
    s_pack.wait_stream(torch.cuda.current_stream())
    ff.ff_pack_to_host(plan, chunks, crcs, h_chunks, h_crcs, slice_chunks, s_pack, s_copy)
    s_copy.synchronize()
    s_pack.synchronize()
    want_buf, want_crcs = oracle.pack(_host_segments(shard)[0], shard.chunk_bytes, threads=4)
    assert np.array_equal(h_chunks.numpy(), want_buf)
    assert np.array_equal(h_crcs.numpy().view(np.uint32), want_crcs)
    assert np.array_equal(chunks.cpu().numpy(), want_buf)       # the device staging holds it too
    assert np.array_equal(_u32(crcs), want_crcs)


# ---- the calls together: a worker's step, a damaged transfer, a newcomer's recovery -----------------

def test_failover_scenario(oracle):
    """Section 3.1, steps 5-6, with this library's pieces: a worker takes an optimizer step that
    snapshots its state; the snapshot reaches a newcomer with a few chunks damaged; the newcomer
    loads what verified, asks for the damaged chunks again and loads those; its state then equals
    the worker's, which equals the oracle's."""
    numels = [30000, 70001, 4096, 123457]
    C = 1 << 16
    worker = wl.param_shard("w", numels, C, 41, DEV, with_grads=True)
    host = [wl.to_numpy_bytes(t) for t in worker.segments]
    params_np = [(host[4 * i].view(np.uint16), host[4 * i + 1].view(np.float32),
                  host[4 * i + 2].view(np.float32), host[4 * i + 3].view(np.float32))
                 for i in range(len(numels))]
    grads_np = [wl.to_numpy_bytes(p.grad).view(np.uint16) for p in worker.params]
    plan = ff.plan_for_shard(worker)
    chunks, crcs, _, _ = ff.alloc_outputs(plan, DEV)
    ff.ff_adam_step_snapshot(plan, [p.grad for p in worker.params], HP, chunks, crcs)
    torch.cuda.synchronize()
    want_buf, want_crcs = oracle.adam_snapshot(params_np, grads_np, host, C, HP)
    assert np.array_equal(chunks.cpu().numpy(), want_buf) and np.array_equal(_u32(crcs), want_crcs)

    # the newcomer: same layout (checked through the layout id), empty tensors
    newcomer = wl.param_shard("n", numels, C, 99, DEV)
    _poison_segments(newcomer)
    plan_n = ff.plan_for_shard(newcomer)
    assert plan_n.layout_id == plan.layout_id and plan_n.num_chunks == plan.num_chunks
    received = chunks.clone()
    damaged = [1, plan.num_chunks // 2, plan.num_chunks - 1]
    for j in damaged:
        received[j * C + 100 + j] ^= 0x10
    _, _, bad, n_bad = ff.alloc_outputs(plan_n, DEV)
    ff.ff_restore_checked(plan_n, plan.layout_id, received, crcs, bad, n_bad,
                          flags=ff.FF_RESTORE_SKIP_BAD)
    torch.cuda.synchronize()
    again = torch.nonzero(bad).flatten().tolist()
    assert again == damaged and int(n_bad.item()) == len(damaged)
    # which tensor ranges are still missing: the spans of the bad chunks hold the poison
    stream = _segments_as_stream(newcomer)
    for j in range(plan.num_chunks):
        first, n, begin, end = plan_n.chunk_span(j)
        if j in damaged:
            assert bool((stream[begin:end] == 0xA5).all())
        else:
            assert np.array_equal(stream[begin:end], want_buf[begin:end])
    # the sender transmits the damaged chunks again
    for j in again:
        received[j * C:(j + 1) * C] = chunks[j * C:(j + 1) * C]
    ff.ff_restore_chunks(plan_n, received, crcs, again, bad, n_bad)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0
    for a, b in zip(newcomer.segments, worker.segments):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
    assert np.array_equal(_segments_as_stream(newcomer), want_buf[:plan.payload_bytes])
