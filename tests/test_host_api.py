"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, validates
arguments, and lays snapshots out as defined.  No kernel runs here."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

from paper_2512_03644_amd import binding as ff
from paper_2512_03644_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "ffsnap.h")).read()
    declared = set(re.findall(r"\b(ff_[a-z0-9_]+)\s*\(", header))
    declared -= {"ff_plan"}
    assert declared == set(ff.EXPORTS)
    L = ff.lib()
    for name in declared:
        assert hasattr(L, name), name


def _host_plan(tensors, chunk, **kw):
    return ff.ff_snapshot_plan(tensors, chunk, flags=ff.FF_PLAN_HOST_ONLY, **kw)


def test_layout_matches_definition_and_oracle_sizes(oracle):
    shard = wl.param_shard("s", [1000, 1, 77, 4096, 33333], 4096, 3, "cpu", tiny_recipe=True)
    plan = ff.plan_for_shard(shard, flags=ff.FF_PLAN_HOST_ONLY)
    n_el = sum(p.master.numel() for p in shard.params)
    assert plan.payload_bytes == 14 * n_el == shard.payload_bytes   # size law, section 4.2
    assert plan.num_chunks == shard.num_chunks == oracle.num_chunks(
        [wl.numpy_alias(t) for t in shard.segments], 4096)
    assert plan.buffer_bytes == plan.num_chunks * 4096 and plan.chunk_bytes == 4096
    assert plan.num_segments == 20 and plan.num_params == 5
    off = 0
    for i, t in enumerate(shard.segments):
        b, e = plan.segment_range(i)
        assert (b, e) == (off, off + t.numel() * t.element_size())
        off = e
    # layout id: CRC32C over (chunk_bytes, nbytes...) little-endian uint64 -- oracle's CRC agrees
    key = np.array([4096] + [t.numel() * t.element_size() for t in shard.segments], dtype="<u8")
    assert plan.layout_id == oracle.crc32c(key.view(np.uint8))
    # razor'd list (master, m, v only): 12 bytes per parameter
    razored = [t for p in shard.params for t in (p.master, p.m, p.v)]
    assert _host_plan(razored, 4096).payload_bytes == 12 * n_el


def test_layout_id_depends_on_sizes_and_chunking():
    a = torch.zeros(100, dtype=torch.float32)
    b = torch.zeros(50, dtype=torch.bfloat16)
    base = _host_plan([a, b], 1024).layout_id
    assert _host_plan([a, b], 2048).layout_id != base
    assert _host_plan([b, a], 1024).layout_id != base
    assert _host_plan([a, b, torch.zeros(0)], 1024).layout_id == base   # empty segment skipped
    assert _host_plan([a.clone(), b.clone()], 1024).layout_id == base   # addresses do not matter


def test_argument_validation():
    a = torch.zeros(64, dtype=torch.float32)
    L = ff.lib()
    out = ctypes.c_void_p()
    segs = ff.make_segments([a])
    H = ff.FF_PLAN_HOST_ONLY

    def plan_status(segs, n, chunk, flags=H):
        return L.ff_snapshot_plan(segs, n, chunk, flags, ctypes.byref(out))

    assert plan_status(segs, 1, 1000) == ff.FF_ERR_INVALID           # not a power of two
    assert plan_status(segs, 1, 512) == ff.FF_ERR_INVALID            # below the minimum
    assert plan_status(segs, 1, 1 << 31) == ff.FF_ERR_INVALID        # above the maximum
    assert plan_status(None, 1, 1024) == ff.FF_ERR_NULL
    assert L.ff_snapshot_plan(segs, 1, 1024, H, None) == ff.FF_ERR_NULL
    assert plan_status(segs, 1, 1024, H | 2) == ff.FF_ERR_INVALID    # unknown flag
    # XCD run lengths: 2^28 workgroups per XCD is the longest a 32-bit launch index allows
    assert plan_status(segs, 1, 1024, H | ff.FF_PLAN_XCD_ORDER(30)) == ff.FF_ERR_INVALID
    for n in (1, 4, 29, 31):
        assert plan_status(segs, 1, 1024, H | ff.FF_PLAN_XCD_ORDER(n)) == ff.FF_OK
        L.ff_plan_destroy(out)
    assert plan_status(segs, 0, 1024) == ff.FF_ERR_EMPTY
    empty = ff.make_segments([torch.zeros(0)])
    assert plan_status(empty, 1, 1024) == ff.FF_ERR_EMPTY
    for field, value, want in (("dtype", 7, ff.FF_ERR_INVALID), ("kind", 9, ff.FF_ERR_INVALID),
                               ("reserved", 1, ff.FF_ERR_INVALID), ("nbytes", 6, ff.FF_ERR_INVALID),
                               ("ptr", None, ff.FF_ERR_NULL),
                               ("ptr", a.data_ptr() + 2, ff.FF_ERR_INVALID)):
        s = ff.make_segments([a])
        setattr(s[0], field, value)
        assert plan_status(s, 1, 1024) == want, field
        assert not out.value
    # a bf16 segment may start on any even address
    s = ff.make_segments([a.view(torch.bfloat16)[1:3]])
    assert plan_status(s, 1, 1024) == ff.FF_OK
    L.ff_plan_destroy(out)
    assert "pointer" in ff.ff_strerror(ff.FF_ERR_NULL) and ff.ff_strerror(0) == "ok"


def test_host_only_plan_refuses_device_work():
    a = torch.zeros(1024, dtype=torch.float32)
    plan = _host_plan([a], 1024)
    L = ff.lib()
    dummy = ctypes.c_void_p(16)
    assert L.ff_pack(plan.handle, dummy, dummy, None) == ff.FF_ERR_HOST_ONLY
    assert L.ff_restore(plan.handle, dummy, dummy, dummy, dummy, 0, None) == ff.FF_ERR_HOST_ONLY
    assert L.ff_pack(None, dummy, dummy, None) == ff.FF_ERR_NULL
    hp = ff.ff_adam_hparams(3e-4, 0.9, 0.95, 1e-8, 0.1, 1)
    ptrs = (ctypes.c_void_p * 1)(16)
    other = ctypes.c_void_p(1 << 40)
    assert L.ff_adam_step_chained(plan.handle, ptrs, ctypes.byref(hp), ctypes.c_float(1.0), None,
                                  other, dummy, dummy, None) == ff.FF_ERR_HOST_ONLY
    assert L.ff_adam_step_chained(None, ptrs, ctypes.byref(hp), ctypes.c_float(1.0), None,
                                  other, dummy, dummy, None) == ff.FF_ERR_NULL
    assert L.ff_adam_step_chained(plan.handle, ptrs, ctypes.byref(hp), ctypes.c_float(1.0), None,
                                  None, dummy, dummy, None) == ff.FF_ERR_NULL
    assert L.ff_plan_segment_range(plan.handle, 5, ctypes.byref(ctypes.c_uint64()),
                                   ctypes.byref(ctypes.c_uint64())) == ff.FF_ERR_INVALID


def test_parameter_groups():
    shard = wl.param_shard("s", [10, 20], 1024, 3, "cpu")
    assert ff.plan_for_shard(shard, flags=ff.FF_PLAN_HOST_ONLY).num_params == 2
    # an incomplete group: the plan still packs, but offers no parameter groups to the fused step
    kinds = [ff.FF_KIND_W16, ff.FF_KIND_MASTER, ff.FF_KIND_M]
    p = shard.params[0]
    plan = _host_plan([p.w16, p.master, p.m], 1024, kinds=kinds, param_ids=[0, 0, 0])
    assert plan.num_params == 0 and plan.payload_bytes == 10 * 10
    # fp16 working weights form groups as well; one plan holds one 16-bit format
    half = wl.param_shard("h", [10, 20], 1024, 3, "cpu", half=torch.float16)
    assert ff.plan_for_shard(half, flags=ff.FF_PLAN_HOST_ONLY).num_params == 2
    kinds = [ff.FF_KIND_W16, ff.FF_KIND_MASTER, ff.FF_KIND_M, ff.FF_KIND_V] * 2
    q = half.params[1]
    both = [p.w16, p.master, p.m, p.v, q.w16, q.master, q.m, q.v]
    assert _host_plan(both, 1024, kinds=kinds, param_ids=[0] * 4 + [1] * 4).num_params == 0
    # an fp32 tensor in the working-weight role is not a group
    assert _host_plan([p.master.clone(), p.master, p.m, p.v], 1024, kinds=kinds[:4],
                      param_ids=[0] * 4).num_params == 0


def test_fold_relations_are_multiples_of_the_generator(oracle):
    # every tap relation in fold_taps.h: x^(32*(S*NE+f)) == sum_k x^(32*(S*e_k+f_k)) mod P,
    # evaluated with the oracle's zero-byte shift (x^(8n) = shift(0x80000000, n))
    text = open(os.path.join(ROOT, "paper_2512_03644_amd", "csrc", "fold_taps.h")).read()
    for body in re.findall(r"struct \w+ \{\n(.*?)\n\};", text, flags=re.S):
        val = {k: int(v) for k, v in re.findall(r"constexpr int (\w+) = (\d+);", body)}
        tabs = {}
        for name, init in re.findall(r"(TAP_[EF])\[NF\]\[NTAP\] = \{(.*)\};", body):
            tabs[name] = [[int(x) for x in row.split(",")] for row in re.findall(r"\{([\d, ]+)\}", init)]
        S, NE, NF, NT = val["STRIDE"], val["NE"], val["NF"], val["NTAP"]
        assert S * 4 == val["ROW_BYTES"] and len(tabs["TAP_E"]) == NF
        for f in range(NF):
            acc = oracle.crc_shift(0x80000000, 4 * (S * NE + f))
            assert len(tabs["TAP_E"][f]) == NT
            for e, c in zip(tabs["TAP_E"][f], tabs["TAP_F"][f]):
                if (e, c) == (255, 255):      # unused slot
                    continue
                assert 0 <= e < NE and 0 <= c < NF
                acc ^= oracle.crc_shift(0x80000000, 4 * (S * e + c))
            assert acc == 0


def test_chunk_span_names_the_segments_a_chunk_covers():
    rng = np.random.default_rng(12)
    sizes = [int(x) for x in rng.integers(1, 900, size=40)]
    tensors = [torch.zeros(n, dtype=torch.float32 if i % 2 else torch.bfloat16)
               for i, n in enumerate(sizes)]
    C = 1024
    plan = _host_plan(tensors, C)
    ranges = [plan.segment_range(i) for i in range(plan.num_segments)]
    for j in range(plan.num_chunks):
        first, n, begin, end = plan.chunk_span(j)
        assert begin == j * C and end == min((j + 1) * C, plan.payload_bytes)
        want = [i for i, (b, e) in enumerate(ranges) if b < end and e > begin]
        assert list(range(first, first + n)) == want
    L = ff.lib()
    z = [ctypes.c_uint64() for _ in range(4)]
    assert L.ff_plan_chunk_span(plan.handle, plan.num_chunks, *[ctypes.byref(x) for x in z]) \
        == ff.FF_ERR_INVALID


def test_checkpoint_razor_rules_and_size_law(oracle):
    shard = wl.param_shard("s", [1000, 77, 4096], 4096, 3, "cpu")
    raw = torch.zeros(10, dtype=torch.float32)
    tensors = [raw] + shard.segments
    kinds = [ff.FF_KIND_RAW] + [ff.FF_KIND_W16, ff.FF_KIND_MASTER, ff.FF_KIND_M, ff.FF_KIND_V] * 3
    names = {ff.FF_KIND_RAW: "raw", ff.FF_KIND_W16: "weight", ff.FF_KIND_MASTER: "optimizer",
             ff.FF_KIND_M: "optimizer", ff.FF_KIND_V: "optimizer"}
    segs = ff.make_segments(tensors, kinds, [0] + [p for p in range(3) for _ in range(4)])
    n_el = sum(p.master.numel() for p in shard.params)
    for d in (1, 2, 8, 64):
        for dist in (False, True):
            uniq = ff.ff_razor_select(segs, len(tensors), d, dist, ff.FF_RAZOR_UNIQUE)
            red = ff.ff_razor_select(segs, len(tensors), d, dist, ff.FF_RAZOR_REDUNDANT)
            assert uniq == oracle.razor_unique([names[k] for k in kinds], d, dist)
            assert sorted(uniq + red) == list(range(len(tensors))) and not set(uniq) & set(red)
            nbytes = sum(tensors[i].numel() * tensors[i].element_size() for i in uniq) - 40
            if d == 1:
                assert nbytes == 14 * n_el
            elif dist:
                assert nbytes == 12 * n_el      # the paper's 12*phi/d per worker
            else:
                assert nbytes == 0
            if uniq:
                plan = _host_plan([tensors[i] for i in uniq], 4096)
                assert plan.payload_bytes == nbytes + 40
    L = ff.lib()
    out = (ctypes.c_uint64 * 16)()
    n = ctypes.c_uint64()
    bad_cfg = ff.ff_razor_config(0, 0)
    assert L.ff_razor_select(segs, 13, ctypes.byref(bad_cfg), 0, out, ctypes.byref(n)) == ff.FF_ERR_INVALID
    ok_cfg = ff.ff_razor_config(2, 1)
    assert L.ff_razor_select(segs, 13, ctypes.byref(ok_cfg), 2, out, ctypes.byref(n)) == ff.FF_ERR_INVALID
    assert L.ff_razor_select(segs, 13, None, 0, out, ctypes.byref(n)) == ff.FF_ERR_NULL


def test_random_layouts_agree_with_the_definition(oracle):
    """Property check over random segment lists: sizes follow the definition, segment ranges tile
    the stream, and every chunk's span names exactly the segments that intersect it."""
    from hypothesis import given, settings, strategies as st

    seg = st.tuples(st.integers(0, 5000), st.sampled_from([torch.bfloat16, torch.float16, torch.float32]))

    @settings(max_examples=60, deadline=None)
    @given(st.lists(seg, min_size=1, max_size=25), st.sampled_from([1024, 2048, 8192, 1 << 16]))
    def check(segs, chunk):
        tensors = [torch.zeros(n, dtype=dt) for n, dt in segs]
        sizes = [t.numel() * t.element_size() for t in tensors]
        total = sum(sizes)
        if total == 0:
            with pytest.raises(ff.FFError) as e:
                _host_plan(tensors, chunk)
            assert e.value.status == ff.FF_ERR_EMPTY
            return
        plan = _host_plan(tensors, chunk)
        assert plan.payload_bytes == total
        assert plan.num_chunks == -(-total // chunk) == oracle.num_chunks(
            [wl.numpy_alias(t) for t in tensors], chunk)
        assert plan.buffer_bytes == plan.num_chunks * chunk
        nonempty = [s for s in sizes if s]
        assert plan.num_segments == len(nonempty)
        ranges, off = [], 0
        for i, s in enumerate(nonempty):
            assert plan.segment_range(i) == (off, off + s)
            ranges.append((off, off + s))
            off += s
        for j in range(plan.num_chunks):
            first, n, begin, end = plan.chunk_span(j)
            assert (begin, end) == (j * chunk, min((j + 1) * chunk, total))
            want = [i for i, (a, b) in enumerate(ranges) if a < end and b > begin]
            assert list(range(first, first + n)) == want

    check()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert run.returncode == 2 and "one GPU" in run.stderr and run.stdout.strip() == ""
