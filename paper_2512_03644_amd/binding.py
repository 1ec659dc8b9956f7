"""ctypes binding of libffsnap.so: the same names as include/ffsnap.h, argument marshalling only.

Tensors are torch tensors (PyTorch supplies device memory and streams, nothing else); every step
of the path runs inside the library's kernels.  If the library has not been built the first call
raises: there is no fallback path.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libffsnap.so")

FF_OK, FF_ERR_NULL, FF_ERR_INVALID, FF_ERR_EMPTY = 0, -1, -2, -3
FF_ERR_NOMEM, FF_ERR_HIP, FF_ERR_HOST_ONLY, FF_ERR_TOO_LARGE, FF_ERR_LAYOUT = -4, -5, -6, -7, -8
FF_CRC32C_NOALLOC_MAX_BYTES = 1 << 36
FF_BF16, FF_F32, FF_F16 = 1, 2, 3
FF_KIND_RAW, FF_KIND_W16, FF_KIND_MASTER, FF_KIND_M, FF_KIND_V = 0, 1, 2, 3, 4
FF_PLAN_HOST_ONLY = 1


def FF_PLAN_TILE_LOG2(n):
    """Plan flag: tile size 2^n bytes (tuning knob; 0 = default)."""
    return (n & 0xFF) << 8


def FF_PLAN_CACHE_HINT(h):
    """Plan flag: bit 0 of h = non-temporal tensor-side accesses, bit 1 = buffer side."""
    return 0x40000 | ((h & 3) << 16)


def FF_PLAN_XCD_ORDER(n):
    """Plan flag: every XCD takes runs of 2^(n-1) workgroup tiles (0 = default, 1..29, 31 = launch
    order)."""
    return (n & 31) << 19

FF_RESTORE_VERIFY_ONLY = 1
FF_RESTORE_SKIP_BAD = 2

EXPORTS = ["ff_snapshot_plan", "ff_plan_destroy", "ff_plan_payload_bytes", "ff_plan_num_chunks",
           "ff_plan_buffer_bytes", "ff_plan_chunk_bytes", "ff_plan_num_segments",
           "ff_plan_num_params", "ff_plan_layout_id", "ff_plan_segment_range",
           "ff_plan_chunk_span", "ff_razor_select", "ff_pack", "ff_pack_to_host", "ff_restore", "ff_restore_checked", "ff_restore_chunks", "ff_adam_step_snapshot",
           "ff_adam_step_snapshot_f16", "ff_adam_step_chained", "ff_crc32c", "ff_crc32c_noalloc",
           "ff_copy_ceiling", "ff_mix_ceiling", "ff_strerror"]


class ff_segment(ctypes.Structure):
    _fields_ = [("ptr", ctypes.c_void_p), ("nbytes", ctypes.c_uint64), ("dtype", ctypes.c_uint32),
                ("kind", ctypes.c_uint32), ("param_id", ctypes.c_uint32),
                ("reserved", ctypes.c_uint32)]


class ff_adam_hparams(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("step", ctypes.c_uint32)]


class ff_razor_config(ctypes.Structure):
    _fields_ = [("dp_degree", ctypes.c_uint32), ("distributed_optimizer", ctypes.c_uint32)]


FF_RAZOR_UNIQUE, FF_RAZOR_REDUNDANT = 0, 1


class FFError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("ffsnap status %d: %s" % (status, text))
        self.status = status


_lib = None


def lib():
    """The loaded C library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libffsnap.so is not built: run paper_2512_03644_amd/build.py "
                               "(there is no fallback implementation)")
        L = ctypes.CDLL(LIB_PATH)
        vp, u64, u32, i32 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int
        L.ff_snapshot_plan.restype = i32
        L.ff_snapshot_plan.argtypes = [ctypes.POINTER(ff_segment), u64, u64, u32,
                                       ctypes.POINTER(vp)]
        L.ff_plan_destroy.restype = None
        L.ff_plan_destroy.argtypes = [vp]
        for name in ("payload_bytes", "num_chunks", "buffer_bytes", "chunk_bytes", "num_segments",
                     "num_params"):
            fn = getattr(L, "ff_plan_" + name)
            fn.restype, fn.argtypes = u64, [vp]
        L.ff_plan_layout_id.restype, L.ff_plan_layout_id.argtypes = u32, [vp]
        L.ff_plan_segment_range.restype = i32
        L.ff_plan_segment_range.argtypes = [vp, u64, ctypes.POINTER(u64), ctypes.POINTER(u64)]
        L.ff_plan_chunk_span.restype = i32
        L.ff_plan_chunk_span.argtypes = [vp, u64] + [ctypes.POINTER(u64)] * 4
        L.ff_restore_chunks.restype = i32
        L.ff_restore_chunks.argtypes = [vp, vp, vp, ctypes.POINTER(u64), u64, vp, vp, u32, vp]
        L.ff_razor_select.restype = i32
        L.ff_razor_select.argtypes = [ctypes.POINTER(ff_segment), u64,
                                      ctypes.POINTER(ff_razor_config), u32, ctypes.POINTER(u64),
                                      ctypes.POINTER(u64)]
        L.ff_pack.restype, L.ff_pack.argtypes = i32, [vp, vp, vp, vp]
        L.ff_pack_to_host.restype = i32
        L.ff_pack_to_host.argtypes = [vp, vp, vp, vp, vp, u64, vp, vp]
        L.ff_restore.restype, L.ff_restore.argtypes = i32, [vp, vp, vp, vp, vp, u32, vp]
        L.ff_restore_checked.restype = i32
        L.ff_restore_checked.argtypes = [vp, u32, vp, vp, vp, vp, u32, vp]
        L.ff_adam_step_snapshot.restype = i32
        L.ff_adam_step_snapshot.argtypes = [vp, ctypes.POINTER(vp),
                                            ctypes.POINTER(ff_adam_hparams), vp, vp, vp]
        L.ff_adam_step_snapshot_f16.restype = i32
        L.ff_adam_step_snapshot_f16.argtypes = [vp, ctypes.POINTER(vp),
                                                ctypes.POINTER(ff_adam_hparams), ctypes.c_float,
                                                vp, vp, vp, vp]
        L.ff_adam_step_chained.restype = i32
        L.ff_adam_step_chained.argtypes = [vp, ctypes.POINTER(vp),
                                           ctypes.POINTER(ff_adam_hparams), ctypes.c_float, vp,
                                           vp, vp, vp, vp]
        L.ff_crc32c.restype, L.ff_crc32c.argtypes = i32, [vp, u64, vp, vp]
        L.ff_crc32c_noalloc.restype, L.ff_crc32c_noalloc.argtypes = i32, [vp, u64, vp, vp]
        L.ff_copy_ceiling.restype, L.ff_copy_ceiling.argtypes = i32, [vp, vp, u64, vp]
        L.ff_mix_ceiling.restype = i32
        L.ff_mix_ceiling.argtypes = [vp, ctypes.POINTER(vp), vp, vp, vp]
        L.ff_strerror.restype, L.ff_strerror.argtypes = ctypes.c_char_p, [i32]
        _lib = L
    return _lib


def ff_strerror(status):
    return lib().ff_strerror(status).decode()


def _check(status):
    if status != FF_OK:
        raise FFError(status, ff_strerror(status))


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


_DTYPES = {torch.bfloat16: FF_BF16, torch.float32: FF_F32, torch.float16: FF_F16}


def make_segments(tensors, kinds=None, param_ids=None):
    """ff_segment array for a list of contiguous bf16/fp32 tensors (stream order)."""
    n = len(tensors)
    arr = (ff_segment * max(n, 1))()
    for i, t in enumerate(tensors):
        if not t.is_contiguous():
            raise ValueError("segment %d is not contiguous" % i)
        arr[i].ptr = t.data_ptr() if t.numel() else None
        arr[i].nbytes = t.numel() * t.element_size()
        arr[i].dtype = _DTYPES[t.dtype]
        arr[i].kind = kinds[i] if kinds is not None else FF_KIND_RAW
        arr[i].param_id = param_ids[i] if param_ids is not None else 0
        arr[i].reserved = 0
    return arr


class Plan:
    """Owns an ff_plan handle; keeps the tensors it points at alive."""

    def __init__(self, handle, keepalive):
        self.handle = handle
        self._keepalive = keepalive

    def destroy(self):
        if self.handle:
            lib().ff_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    payload_bytes = property(lambda s: int(lib().ff_plan_payload_bytes(s.handle)))
    num_chunks = property(lambda s: int(lib().ff_plan_num_chunks(s.handle)))
    buffer_bytes = property(lambda s: int(lib().ff_plan_buffer_bytes(s.handle)))
    chunk_bytes = property(lambda s: int(lib().ff_plan_chunk_bytes(s.handle)))
    num_segments = property(lambda s: int(lib().ff_plan_num_segments(s.handle)))
    num_params = property(lambda s: int(lib().ff_plan_num_params(s.handle)))
    layout_id = property(lambda s: int(lib().ff_plan_layout_id(s.handle)))

    def chunk_span(self, chunk):
        """(first_seg, n_seg, begin, end) of a chunk."""
        v = [ctypes.c_uint64() for _ in range(4)]
        _check(lib().ff_plan_chunk_span(self.handle, chunk, *[ctypes.byref(x) for x in v]))
        return tuple(x.value for x in v)

    def segment_range(self, i):
        b, e = ctypes.c_uint64(), ctypes.c_uint64()
        _check(lib().ff_plan_segment_range(self.handle, i, ctypes.byref(b), ctypes.byref(e)))
        return b.value, e.value


def ff_snapshot_plan(tensors, chunk_bytes, flags=0, kinds=None, param_ids=None, tile_log2=0):
    segs = make_segments(tensors, kinds, param_ids)
    return ff_snapshot_plan_raw(segs, len(tensors), chunk_bytes, flags | (tile_log2 << 8),
                                keepalive=list(tensors))


def ff_snapshot_plan_raw(segs, n_segs, chunk_bytes, flags=0, keepalive=None):
    out = ctypes.c_void_p()
    _check(lib().ff_snapshot_plan(segs, n_segs, chunk_bytes, flags, ctypes.byref(out)))
    return Plan(out, keepalive)


def plan_for_shard(shard, flags=0, tile_log2=0):
    """Plan for a workloads.Shard: parameter groups get their kinds, the rest is RAW."""
    kinds, pids = [], []
    if shard.params:
        for pid, _ in enumerate(shard.params):
            kinds += [FF_KIND_W16, FF_KIND_MASTER, FF_KIND_M, FF_KIND_V]
            pids += [pid] * 4
    else:
        kinds, pids = [FF_KIND_RAW] * len(shard.segments), [0] * len(shard.segments)
    return ff_snapshot_plan(shard.segments, shard.chunk_bytes, flags, kinds, pids, tile_log2)


def ff_razor_select(segs, n_segs, dp_degree, distributed_optimizer, which=FF_RAZOR_UNIQUE):
    """Indices of the unique (or redundant) segments of an ff_segment array."""
    cfg = ff_razor_config(dp_degree, 1 if distributed_optimizer else 0)
    out = (ctypes.c_uint64 * max(n_segs, 1))()
    n = ctypes.c_uint64()
    _check(lib().ff_razor_select(segs, n_segs, ctypes.byref(cfg), which, out, ctypes.byref(n)))
    return [int(out[i]) for i in range(n.value)]


def ff_pack(plan, chunks, crcs, stream=None):
    _check(lib().ff_pack(plan.handle, chunks.data_ptr(), crcs.data_ptr(), _stream_ptr(stream)))


def ff_pack_to_host(plan, chunks, crcs, host_chunks, host_crcs, slice_chunks, pack_stream,
                    copy_stream):
    """host_chunks / host_crcs: CPU tensors (pinned for overlap)."""
    _check(lib().ff_pack_to_host(plan.handle, chunks.data_ptr(), crcs.data_ptr(),
                                 host_chunks.data_ptr(), host_crcs.data_ptr(), slice_chunks,
                                 _stream_ptr(pack_stream), _stream_ptr(copy_stream)))


def ff_restore(plan, chunks, crcs, bad, n_bad, flags=0, stream=None):
    _check(lib().ff_restore(plan.handle, chunks.data_ptr(), crcs.data_ptr(), bad.data_ptr(),
                            n_bad.data_ptr(), flags, _stream_ptr(stream)))


def ff_restore_checked(plan, sender_layout_id, chunks, crcs, bad, n_bad, flags=0, stream=None):
    _check(lib().ff_restore_checked(plan.handle, sender_layout_id, chunks.data_ptr(),
                                    crcs.data_ptr(), bad.data_ptr(), n_bad.data_ptr(), flags,
                                    _stream_ptr(stream)))


def ff_restore_chunks(plan, chunks, crcs, chunk_ids, bad, n_bad, flags=0, stream=None):
    ids = (ctypes.c_uint64 * max(len(chunk_ids), 1))(*[int(c) for c in chunk_ids])
    _check(lib().ff_restore_chunks(plan.handle, chunks.data_ptr(), crcs.data_ptr(), ids,
                                   len(chunk_ids), bad.data_ptr(), n_bad.data_ptr(), flags,
                                   _stream_ptr(stream)))


def ff_adam_step_snapshot(plan, grads, hparams, chunks, crcs, stream=None):
    """grads: list of bf16 device tensors, one per parameter group in ascending param_id;
    hparams: dict(lr, beta1, beta2, eps, weight_decay, step)."""
    ptrs = (ctypes.c_void_p * max(len(grads), 1))(*[g.data_ptr() for g in grads])
    hp = ff_adam_hparams(hparams["lr"], hparams["beta1"], hparams["beta2"], hparams["eps"],
                         hparams["weight_decay"], hparams["step"])
    _check(lib().ff_adam_step_snapshot(plan.handle, ptrs, ctypes.byref(hp), chunks.data_ptr(),
                                       crcs.data_ptr(), _stream_ptr(stream)))


def ff_adam_step_snapshot_f16(plan, grads, hparams, inv_loss_scale, n_nonfinite, chunks, crcs,
                              stream=None):
    """grads: list of fp16 device tensors (gradients of the scaled loss); n_nonfinite: one-element
    int64 device tensor, or None."""
    ptrs = (ctypes.c_void_p * max(len(grads), 1))(*[g.data_ptr() for g in grads])
    hp = ff_adam_hparams(hparams["lr"], hparams["beta1"], hparams["beta2"], hparams["eps"],
                         hparams["weight_decay"], hparams["step"])
    _check(lib().ff_adam_step_snapshot_f16(
        plan.handle, ptrs, ctypes.byref(hp), ctypes.c_float(inv_loss_scale),
        ctypes.c_void_p(n_nonfinite.data_ptr()) if n_nonfinite is not None else None,
        chunks.data_ptr(), crcs.data_ptr(), _stream_ptr(stream)))


def ff_adam_step_chained(plan, grads, hparams, prev_chunks, chunks, crcs, inv_loss_scale=1.0,
                         n_nonfinite=None, stream=None):
    """The step that reads master, m, v from the snapshot `prev_chunks` and writes the new
    snapshot into `chunks`; grads in the plan's 16-bit format."""
    ptrs = (ctypes.c_void_p * max(len(grads), 1))(*[g.data_ptr() for g in grads])
    hp = ff_adam_hparams(hparams["lr"], hparams["beta1"], hparams["beta2"], hparams["eps"],
                         hparams["weight_decay"], hparams["step"])
    _check(lib().ff_adam_step_chained(
        plan.handle, ptrs, ctypes.byref(hp), ctypes.c_float(inv_loss_scale),
        ctypes.c_void_p(n_nonfinite.data_ptr()) if n_nonfinite is not None else None,
        prev_chunks.data_ptr(), chunks.data_ptr(), crcs.data_ptr(), _stream_ptr(stream)))


def ff_crc32c(buf, nbytes, out, stream=None):
    _check(lib().ff_crc32c(buf.data_ptr(), nbytes, out.data_ptr(), _stream_ptr(stream)))


def ff_crc32c_noalloc(buf, nbytes, out, stream=None):
    _check(lib().ff_crc32c_noalloc(buf.data_ptr(), nbytes, out.data_ptr(), _stream_ptr(stream)))


def ff_copy_ceiling(dst, src, nbytes, stream=None):
    _check(lib().ff_copy_ceiling(dst.data_ptr(), src.data_ptr(), nbytes, _stream_ptr(stream)))


def ff_mix_ceiling(plan, grads, prev_chunks, chunks, stream=None):
    """The optimizer steps' loads and stores alone (prev_chunks None: in-place mix; else chained)."""
    ptrs = (ctypes.c_void_p * max(len(grads), 1))(*[g.data_ptr() for g in grads])
    _check(lib().ff_mix_ceiling(plan.handle, ptrs,
                                prev_chunks.data_ptr() if prev_chunks is not None else None,
                                chunks.data_ptr(), _stream_ptr(stream)))


def alloc_outputs(plan, device):
    """(chunks uint8, crcs int32 viewable as uint32, bad int32, n_bad int64) on `device`."""
    chunks = torch.empty(plan.buffer_bytes, dtype=torch.uint8, device=device)
    crcs = torch.empty(plan.num_chunks, dtype=torch.int32, device=device)
    bad = torch.empty(plan.num_chunks, dtype=torch.int32, device=device)
    n_bad = torch.empty(1, dtype=torch.int64, device=device)
    return chunks, crcs, bad, n_bad
