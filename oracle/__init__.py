"""ctypes front end of the CPU oracle (oracle/ffsnap_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  The product package never imports it, and it never imports the
product package.  All arrays are numpy arrays in host memory.
"""
import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ffsnap_oracle.c")
_LIB = os.path.join(_HERE, "libffsnap_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc.  -ffp-contract=off and SSE scalar math keep every fp32
    operation separately rounded."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-msse2",
             "-mfpmath=sse", "-fno-fast-math", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class AdamHParams(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("step", ctypes.c_uint32)]


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        u8p, u32p, u64p = (ctypes.POINTER(ctypes.c_uint8), ctypes.POINTER(ctypes.c_uint32),
                           ctypes.POINTER(ctypes.c_uint64))
        vpp = ctypes.POINTER(ctypes.c_void_p)
        u64, u32 = ctypes.c_uint64, ctypes.c_uint32
        L.orc_init.restype = None
        L.orc_crc_reg.restype = u32
        L.orc_crc_reg.argtypes = [u32, ctypes.c_void_p, u64]
        L.orc_crc32c_bitwise.restype = u32
        L.orc_crc32c_bitwise.argtypes = [ctypes.c_void_p, u64]
        L.orc_crc32c.restype = u32
        L.orc_crc32c.argtypes = [ctypes.c_void_p, u64]
        L.orc_crc_shift.restype = u32
        L.orc_crc_shift.argtypes = [u32, u64]
        L.orc_crc32c_combine.restype = u32
        L.orc_crc32c_combine.argtypes = [u32, u32, u64]
        L.orc_num_chunks.restype = u64
        L.orc_num_chunks.argtypes = [u64p, u64, u64]
        L.orc_pack_chunks.restype = None
        L.orc_pack_chunks.argtypes = [vpp, u64p, u64, u64, ctypes.c_void_p, u32p, u64, u64]
        L.orc_verify_chunks.restype = u64
        L.orc_verify_chunks.argtypes = [ctypes.c_void_p, u32p, u64, u32p, u64, u64]
        L.orc_scatter_segments.restype = None
        L.orc_scatter_segments.argtypes = [vpp, u64p, u64, ctypes.c_void_p, u64, u64]
        L.orc_restore_chunks.restype = u64
        L.orc_restore_chunks.argtypes = [vpp, u64p, u64, u64, ctypes.c_void_p, u32p, u64p, u64,
                                         u32p, ctypes.c_int]
        L.orc_f32_to_bf16.restype = ctypes.c_uint16
        L.orc_f32_to_bf16.argtypes = [ctypes.c_float]
        L.orc_adam_f32.restype = None
        L.orc_adam_f32.argtypes = [u64] + [ctypes.c_void_p] * 5 + [ctypes.POINTER(AdamHParams)]
        L.orc_f16_to_f32_array.restype = None
        L.orc_f16_to_f32_array.argtypes = [u64, ctypes.c_void_p, ctypes.c_void_p]
        L.orc_f32_to_f16_array.restype = None
        L.orc_f32_to_f16_array.argtypes = [u64, ctypes.c_void_p, ctypes.c_void_p]
        L.orc_adam_f32_f16.restype = None
        L.orc_adam_f32_f16.argtypes = ([u64, ctypes.c_void_p, ctypes.c_float] + [ctypes.c_void_p] * 4 +
                                       [ctypes.POINTER(AdamHParams), u64p])
        L.orc_adam_f64.restype = None
        L.orc_adam_f64.argtypes = ([u64] + [ctypes.c_void_p] * 4 + [ctypes.c_double] * 5 + [u32])
        L.orc_init()
        _lib = L
    return _lib


def _bytes_view(a):
    a = np.ascontiguousarray(a)
    return a.view(np.uint8).reshape(-1)


def crc_reg(c, data):
    d = _bytes_view(data)
    return int(lib().orc_crc_reg(c, d.ctypes.data, d.size))


def crc32c_bitwise(data):
    d = _bytes_view(data)
    return int(lib().orc_crc32c_bitwise(d.ctypes.data, d.size))


def crc32c(data):
    d = _bytes_view(data)
    return int(lib().orc_crc32c(d.ctypes.data, d.size))


def crc_shift(c, nbytes):
    return int(lib().orc_crc_shift(c, nbytes))


def crc32c_combine(crc_a, crc_b, len_b):
    return int(lib().orc_crc32c_combine(crc_a, crc_b, len_b))


def _seg_tables(segments):
    """segments: list of contiguous numpy arrays (any dtype).  Returns (keepalive views,
    void* array, uint64 nbytes array)."""
    views = [s.view(np.uint8).reshape(-1) for s in segments]
    for s, v in zip(segments, views):
        assert s.flags["C_CONTIGUOUS"] and v.size == s.nbytes
    ptrs = (ctypes.c_void_p * max(len(views), 1))(*[v.ctypes.data for v in views])
    nbytes = np.array([v.size for v in views], dtype=np.uint64)
    return views, ptrs, nbytes


def num_chunks(segments, chunk_bytes):
    total = sum(int(s.nbytes) for s in segments)
    return (total + chunk_bytes - 1) // chunk_bytes


def _ranges(n, parts):
    parts = max(1, min(parts, n))
    edges = [n * k // parts for k in range(parts + 1)]
    return [(edges[k], edges[k + 1]) for k in range(parts) if edges[k] < edges[k + 1]]


def pack(segments, chunk_bytes, threads=1, chunk_range=None):
    """Returns (buffer uint8[n_chunks*C], crcs uint32[n_chunks]).  threads>1 hands disjoint chunk
    ranges of the same single-threaded C routine to a thread pool (ctypes drops the GIL).
    chunk_range=(j0, j1) fills only those chunks (the rest of the outputs stay zero)."""
    L = lib()
    views, ptrs, nbytes = _seg_tables(segments)
    n = num_chunks(segments, chunk_bytes)
    buf = np.zeros(n * chunk_bytes, dtype=np.uint8)
    crcs = np.zeros(n, dtype=np.uint32)
    j0, j1 = chunk_range if chunk_range is not None else (0, n)
    nb = nbytes.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64))
    cp = crcs.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32))

    def work(r):
        L.orc_pack_chunks(ptrs, nb, len(views), chunk_bytes, buf.ctypes.data, cp,
                          j0 + r[0], j0 + r[1])

    rs = _ranges(j1 - j0, threads)
    if threads <= 1:
        for r in rs:
            work(r)
    else:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(work, rs))
    return buf, crcs


def verify(buffer, crcs, chunk_bytes, threads=1):
    """Returns (bad uint32[n_chunks], n_bad)."""
    L = lib()
    buffer = _bytes_view(buffer)
    crcs = np.ascontiguousarray(crcs, dtype=np.uint32)
    n = buffer.size // chunk_bytes
    assert n * chunk_bytes == buffer.size and crcs.size == n
    bad = np.zeros(n, dtype=np.uint32)
    u32p = ctypes.POINTER(ctypes.c_uint32)

    def work(r):
        return L.orc_verify_chunks(buffer.ctypes.data, crcs.ctypes.data_as(u32p), chunk_bytes,
                                   bad.ctypes.data_as(u32p), r[0], r[1])

    rs = _ranges(n, threads)
    if threads <= 1:
        tot = sum(work(r) for r in rs)
    else:
        with ThreadPoolExecutor(threads) as ex:
            tot = sum(ex.map(work, rs))
    return bad, int(tot)


def restore(segments, chunk_bytes, buffer, crcs, threads=1):
    """Verify all chunks, then overwrite every segment (numpy arrays, in place) from the buffer.
    Returns (bad, n_bad)."""
    L = lib()
    buffer = _bytes_view(buffer)
    views, ptrs, nbytes = _seg_tables(segments)
    assert buffer.size == num_chunks(segments, chunk_bytes) * chunk_bytes
    bad, n_bad = verify(buffer, crcs, chunk_bytes, threads)
    nb = nbytes.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64))

    def work(r):
        L.orc_scatter_segments(ptrs, nb, len(views), buffer.ctypes.data, r[0], r[1])

    rs = _ranges(len(views), threads)
    if threads <= 1:
        for r in rs:
            work(r)
    else:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(work, rs))
    return bad, n_bad


def restore_chunks(segments, chunk_bytes, buffer, crcs, chunk_ids, bad, skip_bad=False):
    """Selective restore of the listed chunks (see orc_restore_chunks).  `bad` is a uint32 array
    of n_chunks entries, updated in place for the listed chunks only.  Returns n_bad."""
    L = lib()
    buffer = _bytes_view(buffer)
    crcs = np.ascontiguousarray(crcs, dtype=np.uint32)
    views, ptrs, nbytes = _seg_tables(segments)
    ids = np.ascontiguousarray(chunk_ids, dtype=np.uint64)
    assert bad.dtype == np.uint32 and bad.size == crcs.size
    u32p, u64p = ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(ctypes.c_uint64)
    return int(L.orc_restore_chunks(ptrs, nbytes.ctypes.data_as(u64p), len(views), chunk_bytes,
                                    buffer.ctypes.data, crcs.ctypes.data_as(u32p),
                                    ids.ctypes.data_as(u64p), ids.size,
                                    bad.ctypes.data_as(u32p), 1 if skip_bad else 0))


def f32_to_bf16(x):
    return int(lib().orc_f32_to_bf16(ctypes.c_float(x)))


def adam_f32(grad_bf16, master, m, v, w16, lr, beta1, beta2, eps, weight_decay, step):
    """In-place fp32 AdamW step.  grad_bf16, w16: uint16 arrays holding bf16 bit patterns;
    master, m, v: float32 arrays."""
    n = master.size
    for a, dt in ((grad_bf16, np.uint16), (w16, np.uint16), (master, np.float32),
                  (m, np.float32), (v, np.float32)):
        assert a.dtype == dt and a.size == n and a.flags["C_CONTIGUOUS"]
    h = AdamHParams(lr, beta1, beta2, eps, weight_decay, step)
    lib().orc_adam_f32(n, grad_bf16.ctypes.data, master.ctypes.data, m.ctypes.data,
                       v.ctypes.data, w16.ctypes.data, ctypes.byref(h))


def f16_to_f32(bits):
    """fp16 bit patterns (uint16 array) -> float32 array."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float32)
    lib().orc_f16_to_f32_array(bits.size, bits.ctypes.data, out.ctypes.data)
    return out


def f32_to_f16(x):
    """float32 array -> fp16 bit patterns (uint16 array), round to nearest even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().orc_f32_to_f16_array(x.size, x.ctypes.data, out.ctypes.data)
    return out


def adam_f32_f16(grad_f16, inv_scale, master, m, v, w16, lr, beta1, beta2, eps, weight_decay, step):
    """In-place fp32 AdamW step for fp16 training with a loss scale.  grad_f16, w16: uint16 arrays
    holding fp16 bit patterns.  Returns the number of non-finite gradient elements."""
    n = master.size
    for a, dt in ((grad_f16, np.uint16), (w16, np.uint16), (master, np.float32),
                  (m, np.float32), (v, np.float32)):
        assert a.dtype == dt and a.size == n and a.flags["C_CONTIGUOUS"]
    h = AdamHParams(lr, beta1, beta2, eps, weight_decay, step)
    bad = ctypes.c_uint64(0)
    lib().orc_adam_f32_f16(n, grad_f16.ctypes.data, ctypes.c_float(inv_scale), master.ctypes.data,
                           m.ctypes.data, v.ctypes.data, w16.ctypes.data, ctypes.byref(h),
                           ctypes.byref(bad))
    return int(bad.value)


def adam_f64(grad, master, m, v, lr, beta1, beta2, eps, weight_decay, step):
    n = master.size
    for a in (grad, master, m, v):
        assert a.dtype == np.float64 and a.size == n and a.flags["C_CONTIGUOUS"]
    lib().orc_adam_f64(n, grad.ctypes.data, master.ctypes.data, m.ctypes.data, v.ctypes.data,
                       lr, beta1, beta2, eps, weight_decay, step)


def adam_snapshot(params, grads_bf16, segments, chunk_bytes, hparams, threads=1):
    """Fused step as the definition states it: update every parameter group in place, then pack
    the (updated) segment list.  params: list of (w16, master, m, v) numpy arrays that alias
    entries of `segments`; grads_bf16: list of uint16 arrays."""
    for (w16, master, m, v), g in zip(params, grads_bf16):
        adam_f32(g, master, m, v, w16, **hparams)
    return pack(segments, chunk_bytes, threads=threads)


def adam_snapshot_f16(params, grads_f16, inv_scale, segments, chunk_bytes, hparams, threads=1):
    """The fp16 variant of adam_snapshot.  Returns (buffer, crcs, n_nonfinite)."""
    bad = 0
    for (w16, master, m, v), g in zip(params, grads_f16):
        bad += adam_f32_f16(g, inv_scale, master, m, v, w16, **hparams)
    buf, crcs = pack(segments, chunk_bytes, threads=threads)
    return buf, crcs, bad


def adam_snapshot_chained(prev_buffer, params, grads, segments, chunk_bytes, hparams,
                          inv_scale=None, threads=1):
    """The step whose optimizer state lives in the snapshots (the paper alternates between its
    two most recent snapshots, section 4.2, and snapshots right after the update, section 6.2):
    master, m and v of every parameter group are first taken out of `prev_buffer` at their
    segments' stream offsets (the stream is the tight concatenation of `segments`); from there on
    it is adam_snapshot (inv_scale None: bf16) or adam_snapshot_f16.  params: (w16, master, m, v)
    numpy arrays aliasing entries of `segments`; master, m, v are overwritten twice here (old
    state, then new), w16 receives the new working weights.  Returns (buffer, crcs, n_nonfinite)."""
    prev = _bytes_view(prev_buffer)
    offset_of, off = {}, 0
    for seg in segments:
        offset_of[seg.__array_interface__["data"][0]] = off
        off += seg.nbytes
    for _, master, m, v in params:
        for arr in (master, m, v):
            o = offset_of[arr.__array_interface__["data"][0]]
            _bytes_view(arr)[:] = prev[o:o + arr.nbytes]
    if inv_scale is None:
        buf, crcs = adam_snapshot(params, grads, segments, chunk_bytes, hparams, threads=threads)
        return buf, crcs, 0
    return adam_snapshot_f16(params, grads, inv_scale, segments, chunk_bytes, hparams,
                             threads=threads)


def razor_unique(kinds, dp_degree, distributed_optimizer):
    """Checkpoint razor (section 4.2), written out as its truth table.  kinds: 'raw', 'weight',
    'optimizer' per segment.  Returns the indices of the unique segments; the rest is redundant.
      rule 1: d > 1                              -> weights redundant
      rule 2: d > 1 and no distributed optimizer -> optimizer states redundant"""
    table = {
        # (d > 1, distributed optimizer): (weights unique, optimizer states unique)
        (False, False): (True, True),
        (False, True): (True, True),
        (True, False): (False, False),
        (True, True): (False, True),
    }
    w_unique, o_unique = table[(dp_degree > 1, bool(distributed_optimizer))]
    keep = {"raw": True, "weight": w_unique, "optimizer": o_unique}
    return [i for i, k in enumerate(kinds) if keep[k]]
