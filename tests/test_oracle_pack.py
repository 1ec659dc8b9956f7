"""Pins for the oracle's pack / verify / restore: library concatenation, round trip, poison,
guard bands, corruption, the size law of section 4.2."""
import numpy as np
import pytest
import torch

from gf2ref import crc32c_by_division
from paper_2512_03644_amd import workloads as wl


def _np_segments(shard):
    return [wl.numpy_alias(t) for t in shard.segments]


def _small_param_shard(chunk=4096, seed=11):
    numels = [int(x) for x in np.random.default_rng(seed).integers(1, 3000, size=9)]
    return wl.param_shard("small", numels, chunk, seed, "cpu", tiny_recipe=True)


def test_pack_is_concatenation_with_zero_tail(oracle):
    shard = _small_param_shard()
    segs = _np_segments(shard)
    buf, crcs = oracle.pack(segs, shard.chunk_bytes)
    stream = np.concatenate([s.view(np.uint8).reshape(-1) for s in segs])
    n = shard.num_chunks
    assert buf.size == n * shard.chunk_bytes and crcs.size == n
    assert np.array_equal(buf[:stream.size], stream)
    assert not buf[stream.size:].any() and buf.size - stream.size < shard.chunk_bytes
    # CRC covers the whole chunk including the zero tail of the last one
    for j in (0, n // 2, n - 1):
        chunk = buf[j * shard.chunk_bytes:(j + 1) * shard.chunk_bytes]
        assert int(crcs[j]) == crc32c_by_division(chunk.tobytes())


def test_size_law(oracle):
    # 12 bytes per parameter for fp32 master + m + v (section 4.2), 14 with the bf16 weights
    shard = _small_param_shard()
    n_el = sum(p.master.numel() for p in shard.params)
    assert shard.payload_bytes == 14 * n_el
    razored = [wl.numpy_alias(t) for p in shard.params for t in (p.master, p.m, p.v)]
    assert sum(a.nbytes for a in razored) == 12 * n_el
    assert sum(wl.llama7b_dp8_numels()) * 14 == 11791761408
    assert sum(wl.llama70b_dp64_numels()) * 14 == 15433334784
    assert len(wl.llama7b_dp8_numels()) == 226 and len(wl.llama70b_dp64_numels()) == 562


def test_chunk_range_and_threads(oracle):
    shard = _small_param_shard(chunk=2048)
    segs = _np_segments(shard)
    buf, crcs = oracle.pack(segs, shard.chunk_bytes)
    buf4, crcs4 = oracle.pack(segs, shard.chunk_bytes, threads=4)
    assert np.array_equal(buf, buf4) and np.array_equal(crcs, crcs4)
    j0, j1 = 3, 7
    pb, pc = oracle.pack(segs, shard.chunk_bytes, chunk_range=(j0, j1))
    C = shard.chunk_bytes
    assert np.array_equal(pb[j0 * C:j1 * C], buf[j0 * C:j1 * C])
    assert np.array_equal(pc[j0:j1], crcs[j0:j1])
    assert not pb[:j0 * C].any() and not pb[j1 * C:].any()


def test_empty_segments_are_skipped(oracle):
    a = np.arange(10, dtype=np.float32)
    e = np.zeros(0, dtype=np.float32)
    b = np.arange(7, dtype=np.uint16)
    buf1, c1 = oracle.pack([a, e, b, e], 1024)
    buf2, c2 = oracle.pack([a, b], 1024)
    assert np.array_equal(buf1, buf2) and np.array_equal(c1, c2)


def test_restore_round_trip_into_poison(oracle):
    shard = _small_param_shard()
    segs = _np_segments(shard)
    want = [s.copy() for s in segs]
    buf, crcs = oracle.pack(segs, shard.chunk_bytes)
    for s in segs:
        s.view(np.uint8)[...] = 0xA5
    bad, n_bad = oracle.restore(segs, shard.chunk_bytes, buf, crcs, threads=3)
    assert n_bad == 0 and not bad.any()
    for s, w in zip(segs, want):
        assert np.array_equal(s.view(np.uint8), w.view(np.uint8))


def test_restore_leaves_gaps_untouched(oracle):
    lay = wl.fragmented_layout(seed=5, n_tensors=200, mu=5.0, sigma=2.0, max_numel=5000)
    shard = wl.fragmented_shard(lay, 4096, seed=5)
    arena = shard.arena.numpy()
    segs = _np_segments(shard)
    # misalignment really is exercised
    assert len({off % 16 for off, _ in shard.spans}) > 4
    buf, crcs = oracle.pack(segs, shard.chunk_bytes)
    stream = np.concatenate([arena[o:o + n] for o, n in shard.spans])
    assert np.array_equal(buf[:stream.size], stream)
    before = arena.copy()
    mask = np.zeros(arena.size, dtype=bool)
    for o, n in shard.spans:
        mask[o:o + n] = True
        arena[o:o + n] = 0xA5
    bad, n_bad = oracle.restore(segs, shard.chunk_bytes, buf, crcs)
    assert n_bad == 0
    assert np.array_equal(arena[mask], before[mask])
    assert np.array_equal(arena[~mask], before[~mask])


def test_corruption_is_flagged_exactly_and_data_still_written(oracle):
    shard = _small_param_shard(chunk=1024, seed=12)
    segs = _np_segments(shard)
    buf, crcs = oracle.pack(segs, shard.chunk_bytes)
    n = shard.num_chunks
    hits = wl.corrupt_chunks(n, shard.chunk_bytes, seed=3, fraction=0.1)
    dirty = buf.copy()
    for c, off, bit in hits:
        dirty[c * shard.chunk_bytes + off] ^= 1 << bit
    bad, n_bad = oracle.restore(segs, shard.chunk_bytes, dirty, crcs)
    assert n_bad == len(hits) and sorted(np.nonzero(bad)[0]) == [c for c, _, _ in hits]
    got = np.concatenate([s.view(np.uint8).reshape(-1) for s in segs])
    assert np.array_equal(got, dirty[:got.size])          # bad chunks are scattered too
    # a flipped bit in the CRC array flags that chunk as well
    c2 = crcs.copy()
    c2[n - 1] ^= 1 << 17
    bad, n_bad = oracle.restore(segs, shard.chunk_bytes, buf, c2)
    assert n_bad == 1 and bad[n - 1] == 1


def test_swapped_chunks_are_detected(oracle):
    shard = _small_param_shard(chunk=1024, seed=13)
    segs = _np_segments(shard)
    buf, crcs = oracle.pack(segs, shard.chunk_bytes)
    C = shard.chunk_bytes
    sw = buf.copy()
    sw[0:C], sw[C:2 * C] = buf[C:2 * C], buf[0:C]
    bad, n_bad = oracle.verify(sw, crcs, C)
    assert n_bad == 2 and bad[0] == 1 and bad[1] == 1


# ---- selective restore ------------------------------------------------------------------------------

def _poison(segs):
    for s in segs:
        s.view(np.uint8)[...] = 0xA5


def _stream(segs):
    return np.concatenate([s.view(np.uint8).reshape(-1) for s in segs])


def test_restore_chunks_of_all_chunks_is_restore(oracle):
    shard = _small_param_shard(chunk=2048, seed=21)
    segs = _np_segments(shard)
    buf, crcs = oracle.pack(segs, shard.chunk_bytes)
    n = shard.num_chunks
    _poison(segs)
    bad = np.full(n, 7, dtype=np.uint32)
    assert oracle.restore_chunks(segs, shard.chunk_bytes, buf, crcs, np.arange(n), bad) == 0
    assert not bad.any()
    assert np.array_equal(_stream(segs), buf[:shard.payload_bytes])


def test_restore_chunks_touches_only_the_listed_chunks(oracle):
    shard = _small_param_shard(chunk=1024, seed=22)
    segs = _np_segments(shard)
    buf, crcs = oracle.pack(segs, shard.chunk_bytes)
    n, C, N = shard.num_chunks, shard.chunk_bytes, shard.payload_bytes
    ids = np.array([1, 4, n - 1], dtype=np.uint64)
    _poison(segs)
    bad = np.full(n, 7, dtype=np.uint32)
    assert oracle.restore_chunks(segs, C, buf, crcs, ids, bad) == 0
    got = _stream(segs)
    inside = np.zeros(N, dtype=bool)
    for j in ids:
        inside[int(j) * C:min((int(j) + 1) * C, N)] = True
    assert np.array_equal(got[inside], buf[:N][inside])
    assert np.all(got[~inside] == 0xA5)                     # everything else keeps the poison
    assert np.all(bad[ids.astype(int)] == 0)
    assert np.all(np.delete(bad, ids.astype(int)) == 7)     # unlisted entries of bad[] untouched


def test_restore_chunks_skip_bad(oracle):
    shard = _small_param_shard(chunk=1024, seed=23)
    segs = _np_segments(shard)
    buf, crcs = oracle.pack(segs, shard.chunk_bytes)
    n, C, N = shard.num_chunks, shard.chunk_bytes, shard.payload_bytes
    dirty = buf.copy()
    dirty[2 * C + 17] ^= 0x10
    dirty[5 * C + 900] ^= 0x01
    ids = np.array([0, 2, 3, 5], dtype=np.uint64)
    for skip in (False, True):
        _poison(segs)
        bad = np.zeros(n, dtype=np.uint32)
        assert oracle.restore_chunks(segs, C, dirty, crcs, ids, bad, skip_bad=skip) == 2
        assert list(np.nonzero(bad)[0]) == [2, 5]
        got = _stream(segs)
        for j in (0, 3):
            assert np.array_equal(got[j * C:(j + 1) * C], dirty[j * C:(j + 1) * C])
        for j in (2, 5):
            piece = got[j * C:min((j + 1) * C, N)]
            if skip:
                assert np.all(piece == 0xA5)               # destinations left as they were
            else:
                assert np.array_equal(piece, dirty[j * C:min((j + 1) * C, N)])
