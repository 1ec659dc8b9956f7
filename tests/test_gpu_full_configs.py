"""GPU parity at the full sizes of the five configurations, in the launch configuration the bench
times.  Every chunk of every snapshot -- bytes and CRC -- and every element of the optimizer state
is compared with the CPU oracle (run on all host cores over windows of chunks, which bounds the host
memory); round trips, fused == unfused and the exact corruption set are checked on top."""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from paper_2512_03644_amd import binding as ff
from paper_2512_03644_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
CORES = max(1, min(16, len(os.sched_getaffinity(0))))
WINDOW_BYTES = 1 << 30          # chunks compared per round trip to the host


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


def _host_copy(tensors):
    return [wl.to_numpy_bytes(t) for t in tensors]


def _check_all_chunks(oracle, plan, host_segments, chunks, crcs):
    """Every chunk of the device buffer and every CRC against oracle.pack of the host copies of
    the segments, window by window; stops at the first chunk that differs."""
    C, n = plan.chunk_bytes, plan.num_chunks
    assert sum(h.size for h in host_segments) == plan.payload_bytes
    crcs_h = _u32(crcs)
    step = max(1, WINDOW_BYTES // C)
    for j0 in range(0, n, step):
        j1 = min(n, j0 + step)
        want_buf, want_crcs = oracle.pack(host_segments, C, threads=CORES, chunk_range=(j0, j1))
        got = chunks[j0 * C:j1 * C].cpu().numpy()
        want = want_buf[j0 * C:j1 * C]
        if not np.array_equal(got, want):
            diff = np.flatnonzero(got.reshape(j1 - j0, C) != want.reshape(j1 - j0, C))
            raise AssertionError("chunk %d differs from the oracle at byte %d"
                                 % (j0 + diff[0] // C, diff[0] % C))
        if not np.array_equal(crcs_h[j0:j1], want_crcs[j0:j1]):
            j = j0 + int(np.flatnonzero(crcs_h[j0:j1] != want_crcs[j0:j1])[0])
            raise AssertionError("crc of chunk %d: %08x, oracle %08x"
                                 % (j, int(crcs_h[j]), int(want_crcs[j])))
        del want_buf, got, want


def _oracle_update_all(oracle, shard, hp, inv_scale=None):
    """The oracle's optimizer step on host copies of every parameter group (a thread per group;
    the C routine itself is single-threaded).  Returns the host segments, updated in place."""
    host = _host_copy(shard.segments)
    grads = [wl.to_numpy_bytes(p.grad).view(np.uint16) for p in shard.params]

    def upd(i):
        w16, master, m, v = (host[4 * i].view(np.uint16), host[4 * i + 1].view(np.float32),
                             host[4 * i + 2].view(np.float32), host[4 * i + 3].view(np.float32))
        if inv_scale is None:
            oracle.adam_f32(grads[i], master, m, v, w16, **hp)
            return 0
        return oracle.adam_f32_f16(grads[i], inv_scale, master, m, v, w16, **hp)

    with ThreadPoolExecutor(CORES) as ex:
        nonfinite = sum(ex.map(upd, range(len(shard.params))))
    return host, nonfinite


def _check_all_tensors(tensors, host):
    for i, (t, h) in enumerate(zip(tensors, host)):
        if not np.array_equal(wl.to_numpy_bytes(t), h):
            raise AssertionError("segment %d differs from the oracle" % i)


def test_config2_llama7b_pack_restore(oracle):
    shard = wl.config_llama7b(DEV)
    plan = ff.plan_for_shard(shard)
    assert plan.payload_bytes == 11791761408 and plan.num_chunks == 2812
    assert plan.num_segments == 904
    chunks, crcs, bad, n_bad = ff.alloc_outputs(plan, DEV)
    chunks.fill_(0xA5)
    ff.ff_pack(plan, chunks, crcs)
    torch.cuda.synchronize()
    host = _host_copy(shard.segments)
    _check_all_chunks(oracle, plan, host, chunks, crcs)
    del host
    # zero tail of the last chunk
    assert not bool(chunks[plan.payload_bytes:].any())
    # round trip into poisoned tensors
    saved = [t.clone() for t in shard.segments]
    for t in shard.segments:
        t.view(torch.uint8).fill_(0xA5)
    ff.ff_restore(plan, chunks, crcs, bad, n_bad)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0 and not bool(bad.any())
    for t, s in zip(shard.segments, saved):
        assert torch.equal(t.view(torch.uint8), s.view(torch.uint8))


def test_config3_fragmented_full(oracle):
    shard = wl.config_fragmented(DEV)
    plan = ff.plan_for_shard(shard)
    assert plan.num_segments == 20000
    chunks, crcs, bad, n_bad = ff.alloc_outputs(plan, DEV)
    chunks.fill_(0xA5)
    ff.ff_pack(plan, chunks, crcs)
    torch.cuda.synchronize()
    arena = shard.arena.cpu().numpy()
    host = [arena[o:o + n] for o, n in shard.spans]
    want_buf, want_crcs = oracle.pack(host, shard.chunk_bytes, threads=16)
    assert np.array_equal(_u32(crcs), want_crcs)
    got = chunks.cpu().numpy()
    assert np.array_equal(got, want_buf)
    del got, want_buf
    # restore into poisoned segments; the gaps of the arena must not change
    before = shard.arena.clone()
    for o, n in shard.spans:
        shard.arena[o:o + n] = 0xA5
    ff.ff_restore(plan, chunks, crcs, bad, n_bad)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0
    assert torch.equal(shard.arena, before)


def test_config4_fused_adam_full(oracle):
    shard = wl.config_llama7b(DEV, with_grads=True)
    plan = ff.plan_for_shard(shard)
    hp = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=1000)
    # the oracle's step on host copies taken before the in-place update, all 226 groups
    host, _ = _oracle_update_all(oracle, shard, hp)
    chunks, crcs, bad, n_bad = ff.alloc_outputs(plan, DEV)
    chunks.fill_(0xA5)
    ff.ff_adam_step_snapshot(plan, [p.grad for p in shard.params], hp, chunks, crcs)
    torch.cuda.synchronize()
    # every element of w16, master, m, v bit for bit (which implies the 1e-6 acceptance bound;
    # that bound is also written out on one group)
    _check_all_tensors(shard.segments, host)
    got = shard.params[5].master.cpu().numpy().astype(np.float64)
    ref = host[4 * 5 + 1].view(np.float32).astype(np.float64)
    assert np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1.1754944e-38)) <= 1e-6
    # bf16 weights are the exact rounding of the fp32 masters the GPU produced
    for p in shard.params[::17]:
        assert torch.equal(p.w16, p.master.to(torch.bfloat16))
    # the snapshot: every chunk and CRC against the oracle's pack of its updated state
    _check_all_chunks(oracle, plan, host, chunks, crcs)
    del host
    # fused == unfused: packing the in-place result reproduces chunks and CRCs bit for bit
    chunks2, crcs2, _, _ = ff.alloc_outputs(plan, DEV)
    ff.ff_pack(plan, chunks2, crcs2)
    torch.cuda.synchronize()
    assert torch.equal(crcs, crcs2)
    assert torch.equal(chunks, chunks2)


def test_config4_fused_adam_full_fp16(oracle):
    """The same shard in fp16 with a loss scale of 65536 (the paper's models train in fp16)."""
    scale = 65536.0
    shard = wl.config_llama7b(DEV, with_grads=True, half=torch.float16, loss_scale=scale)
    plan = ff.plan_for_shard(shard)
    hp = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=1000)
    inv = float(np.float32(1.0 / scale))
    host, want_nonfinite = _oracle_update_all(oracle, shard, hp, inv_scale=inv)
    chunks, crcs, bad, n_bad = ff.alloc_outputs(plan, DEV)
    n_nonfinite = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    ff.ff_adam_step_snapshot_f16(plan, [p.grad for p in shard.params], hp, inv, n_nonfinite,
                                 chunks, crcs)
    torch.cuda.synchronize()
    # N(0, 1e-3) * 65536 has sigma 65.5: an fp16 overflow would be a 1000-sigma event
    assert int(n_nonfinite.item()) == want_nonfinite == 0
    _check_all_tensors(shard.segments, host)
    for p in shard.params[::17]:
        assert torch.equal(p.w16, p.master.to(torch.float16))
    _check_all_chunks(oracle, plan, host, chunks, crcs)
    del host
    chunks2, crcs2, _, _ = ff.alloc_outputs(plan, DEV)
    ff.ff_pack(plan, chunks2, crcs2)
    torch.cuda.synchronize()
    assert torch.equal(crcs, crcs2)
    assert torch.equal(chunks, chunks2)


def test_config4_chained_step_full(oracle):
    """Config 4 with the optimizer state kept in the snapshots: the step reads snapshot A and writes
    snapshot B.  All of B and of the working weights against the oracle, the tensors the step must
    not touch, and B == the in-place step run on tensors loaded from A."""
    shard = wl.config_llama7b(DEV, with_grads=True)
    plan = ff.plan_for_shard(shard)
    hp = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=1000)
    grads = [p.grad for p in shard.params]
    a, crcs_a, bad, n_bad = ff.alloc_outputs(plan, DEV)
    b, crcs_b, _, _ = ff.alloc_outputs(plan, DEV)
    ff.ff_pack(plan, a, crcs_a)
    # A holds the tensors' state, so the oracle's step on the tensors' host copies is the
    # definition's "take master, m, v out of A, then update, then pack"
    host, _ = _oracle_update_all(oracle, shard, hp)
    for p in shard.params:
        for t in (p.master, p.m, p.v):
            t.view(torch.int32).fill_(0x7FC00BAD)
    b.fill_(0xA5)
    ff.ff_adam_step_chained(plan, grads, hp, a, b, crcs_b)
    torch.cuda.synchronize()
    for i, p in enumerate(shard.params):
        assert np.array_equal(wl.to_numpy_bytes(p.w16), host[4 * i]), i
        for t in (p.master, p.m, p.v):
            assert bool((t.view(torch.int32) == 0x7FC00BAD).all()), i
    _check_all_chunks(oracle, plan, host, b, crcs_b)
    del host
    # the same step in place, on tensors loaded from snapshot A
    ff.ff_restore(plan, a, crcs_a, bad, n_bad)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0
    c, crcs_c = a, crcs_a                      # A is no longer needed: reuse its memory
    ff.ff_adam_step_snapshot(plan, grads, hp, c, crcs_c)
    torch.cuda.synchronize()
    assert torch.equal(crcs_b, crcs_c)
    assert torch.equal(b, c)


def test_config5_llama70b_verified_restore(oracle):
    shard = wl.config_llama70b(DEV)
    plan = ff.plan_for_shard(shard)
    assert plan.payload_bytes == 15433334784 and plan.num_chunks == 1840
    assert plan.num_segments == 2248
    C = plan.chunk_bytes
    chunks, crcs, bad, n_bad = ff.alloc_outputs(plan, DEV)
    ff.ff_pack(plan, chunks, crcs)
    torch.cuda.synchronize()
    host = _host_copy(shard.segments)
    _check_all_chunks(oracle, plan, host, chunks, crcs)
    del host
    hits = wl.corrupt_chunks(plan.num_chunks, C)
    assert len(hits) == 18
    for c, off, bit in hits:
        chunks[c * C + off] ^= (1 << bit)
    saved = [t.clone() for t in shard.segments]
    for t in shard.segments:
        t.view(torch.uint8).fill_(0xA5)
    ff.ff_restore(plan, chunks, crcs, bad, n_bad)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 18
    assert sorted(torch.nonzero(bad).flatten().tolist()) == [c for c, _, _ in hits]
    # the oracle's verdict on the whole corrupted buffer, chunk for chunk
    crcs_h, got_bad = _u32(crcs), _u32(bad)
    step = max(1, WINDOW_BYTES // C)
    total = 0
    for j0 in range(0, plan.num_chunks, step):
        j1 = min(plan.num_chunks, j0 + step)
        wb, wn = oracle.verify(chunks[j0 * C:j1 * C].cpu().numpy(), crcs_h[j0:j1], C, threads=CORES)
        assert np.array_equal(wb, got_bad[j0:j1]), j0
        total += wn
    assert total == 18
    # everything outside the flipped bits round-trips: exactly one differing byte per flip that
    # fell into the payload
    expected = sum(1 for c, off, _ in hits if c * C + off < plan.payload_bytes)
    diff = 0
    for t, s in zip(shard.segments, saved):
        diff += int((t.view(torch.uint8) != s.view(torch.uint8)).sum().item())
    assert diff == expected
