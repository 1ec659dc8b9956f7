"""Seeded synthetic inputs: layouts and values of one worker's training state.

This module only draws numbers and lays tensors out; it holds none of the snapshot method's
arithmetic (no CRC, no packing, no optimizer math) and is the one piece shared by the GPU path's
tests/bench and the CPU oracle's tests.  The shards take the shapes and sizes of Llama-class
models (the paper trains GPT-2 2.7B, LLaMA3-8B, LLaMA2-13B and LLaMA3-70B, section 7.1, table 4)
and stand in for them: the path moves bytes, so only state size and tensor layout matter.

A worker's unique state under data parallelism is the fp32 master weights plus Adam m and v,
12 bytes per parameter (section 4.2); the shards here add the bf16 weights, 14 bytes per
parameter, in parameter-major stream order [w16, master, m, v].
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

SEED_BASE = 25120364

MiB = 1 << 20


@dataclass
class ParamGroup:
    w16: torch.Tensor      # bf16
    master: torch.Tensor   # fp32
    m: torch.Tensor        # fp32
    v: torch.Tensor        # fp32
    grad: Optional[torch.Tensor] = None  # bf16, read-only, never part of the snapshot


@dataclass
class Shard:
    name: str
    chunk_bytes: int
    segments: List[torch.Tensor]                  # stream order
    params: List[ParamGroup] = field(default_factory=list)
    arena: Optional[torch.Tensor] = None          # backing store when segments are carved out
    spans: Optional[list] = None                  # (byte offset in arena, nbytes) per segment

    @property
    def payload_bytes(self):
        return sum(t.numel() * t.element_size() for t in self.segments)

    @property
    def num_chunks(self):
        return (self.payload_bytes + self.chunk_bytes - 1) // self.chunk_bytes


# ---- layouts (element counts only) ----------------------------------------------------------

def tiny_numels(seed=SEED_BASE + 1, n_params=64, lo=1024, hi=65536):
    rng = np.random.default_rng(seed)
    return [int(x) for x in rng.integers(lo, hi, size=n_params, endpoint=True)]


def llama_numels(layers, hidden, ffn, kv_dim, vocab, dp):
    """Per-worker element counts: a 1/dp contiguous slice of every weight matrix, in model
    order embed, then per layer q, k, v, o, gate, up, down, then lm_head."""
    def part(rows, cols):
        assert (rows * cols) % dp == 0
        return rows * cols // dp
    out = [part(vocab, hidden)]
    for _ in range(layers):
        out += [part(hidden, hidden), part(hidden, kv_dim), part(hidden, kv_dim),
                part(hidden, hidden), part(hidden, ffn), part(hidden, ffn), part(ffn, hidden)]
    out.append(part(vocab, hidden))
    return out


def llama7b_dp8_numels():
    return llama_numels(32, 4096, 11008, 4096, 32000, 8)


def llama70b_dp64_numels():
    return llama_numels(80, 8192, 28672, 1024, 128256, 64)


def fragmented_layout(seed=SEED_BASE + 3, n_tensors=20000, mu=9.0, sigma=2.0, max_numel=4 * MiB):
    """(numel, itemsize, misalignment) per tensor: lognormal sizes clipped to [1, max_numel],
    bf16 or fp32 with probability 1/2, start address modulo 16 uniform over the multiples of
    the element size."""
    rng = np.random.default_rng(seed)
    numel = np.clip(np.floor(rng.lognormal(mu, sigma, size=n_tensors)), 1, max_numel).astype(np.int64)
    itemsize = np.where(rng.random(n_tensors) < 0.5, 2, 4).astype(np.int64)
    mis = (rng.integers(0, 16, size=n_tensors) // itemsize) * itemsize
    return [(int(n), int(s), int(a)) for n, s, a in zip(numel, itemsize, mis)]


# ---- values -----------------------------------------------------------------------------------

def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _normal(n, std, gen, device):
    return torch.empty(n, dtype=torch.float32, device=device).normal_(0.0, std, generator=gen)


def param_shard(name, numels, chunk_bytes, seed, device="cpu", with_grads=False,
                tiny_recipe=False, half=torch.bfloat16, loss_scale=1.0):
    """Parameter-major shard.  tiny_recipe: weight, master, m, v each ~N(0, 0.02) (the small
    correctness configuration).  Otherwise the training-like recipe: master ~N(0, 0.02),
    w16 = half(master), m ~N(0, 1e-3), v = N(0, 1e-3)^2 >= 0, grads ~N(0, 1e-3) * loss_scale in
    the 16-bit format `half` (bf16, or fp16 for the loss-scaled variant)."""
    gen = _gen(device, seed)
    segs, params = [], []
    for n in numels:
        master = _normal(n, 0.02, gen, device)
        if tiny_recipe:
            w16 = _normal(n, 0.02, gen, device).to(half)
            m = _normal(n, 0.02, gen, device)
            v = _normal(n, 0.02, gen, device)
        else:
            w16 = master.to(half)
            m = _normal(n, 1e-3, gen, device)
            v = _normal(n, 1e-3, gen, device).square_()
        grad = (_normal(n, 1e-3, gen, device) * loss_scale).to(half) if with_grads else None
        params.append(ParamGroup(w16, master, m, v, grad))
        segs += [w16, master, m, v]
    return Shard(name, chunk_bytes, segs, params)


def fragmented_shard(layout, chunk_bytes, seed, device="cpu", name="fragmented", max_gap=64):
    """All tensors carved from one byte arena at running offsets; a random gap before each one
    places its start at the requested misalignment.  Arena and gaps hold random bytes, so a
    write outside a segment is visible."""
    rng = np.random.default_rng(seed)
    spans, pos = [], 0
    for numel, itemsize, mis in layout:
        pos += int(rng.integers(0, max_gap // 16 + 1)) * 16
        pos = (pos + 15) // 16 * 16 + mis
        spans.append((pos, numel * itemsize))
        pos += numel * itemsize
    arena_bytes = (pos + 15) // 16 * 16 + 16
    gen = _gen(device, seed)
    arena = torch.empty(arena_bytes, dtype=torch.uint8, device=device)
    # random_ fills whole 64-bit words quickly; view the arena as int64
    arena.view(torch.int64).random_(generator=gen)
    segs = []
    for (off, nbytes), (numel, itemsize, _) in zip(spans, layout):
        raw = arena[off:off + nbytes]
        segs.append(raw.view(torch.bfloat16 if itemsize == 2 else torch.float32))
    return Shard(name, chunk_bytes, segs, [], arena, spans)


# ---- the five configurations ------------------------------------------------------------------

def config_tiny(device="cpu"):
    return param_shard("tiny-64", tiny_numels(), 1 * MiB, SEED_BASE + 1, device, tiny_recipe=True)


def config_llama7b(device, with_grads=False, half=torch.bfloat16, loss_scale=1.0):
    return param_shard("llama7b-dp8", llama7b_dp8_numels(), 4 * MiB,
                       SEED_BASE + (4 if with_grads else 2), device, with_grads=with_grads,
                       half=half, loss_scale=loss_scale)


def config_fragmented(device="cpu", n_tensors=20000, max_numel=4 * MiB):
    lay = fragmented_layout(SEED_BASE + 3, n_tensors=n_tensors, max_numel=max_numel)
    return fragmented_shard(lay, 4 * MiB, SEED_BASE + 3, device)


# Variants of the fragmented configuration that take its cost apart: the same 20,000 sizes with
# sizes and starts rounded to various grids, and uniform layouts that put every tile on one path
# of the tile kernels.  name -> (what it is, layout builder, largest gap between tensors)
def _rounded(grid, mis=lambda a: 0):
    """The fragmented layout with every size in bytes rounded up to a multiple of `grid` (to the
    nearest multiple, at least one, for the tile-sized grid) and the misalignment mapped by `mis`."""
    def build():
        out = []
        for n, s, a in fragmented_layout(SEED_BASE + 3):
            nbytes = n * s
            if grid >= 1024:
                nbytes = max(grid, (nbytes + grid // 2) // grid * grid)
            else:
                nbytes = (nbytes + grid - 1) // grid * grid
            out.append((nbytes // s, s, mis(a)))
        return out
    return build


LAYOUT_VARIANTS = {
    "fragmented-tiles": ("sizes rounded to whole 32 KiB tiles, tensors back to back",
                         _rounded(32768), 0),
    "fragmented-16": ("sizes and starts rounded to 16 bytes", _rounded(16), 64),
    "fragmented-16-off4": ("sizes rounded to 16 bytes, starts off by multiples of 4 bytes",
                           _rounded(16, mis=lambda a: a // 4 * 4), 64),
    "fragmented-16-off2": ("sizes rounded to 16 bytes, starts off by multiples of 2 bytes",
                           _rounded(16, mis=lambda a: a), 64),
    "tensors-32k": ("100,000 tensors of 32 KiB back to back", lambda: [(8192, 4, 0)] * 100000, 0),
    "tensors-32k-gaps": ("100,000 tensors of 32 KiB, gaps of 0-64 bytes in steps of 16",
                         lambda: [(8192, 4, 0)] * 100000, 64),
    "tensors-33k": ("100,000 tensors of 33 KiB: every tile touches two tensors",
                    lambda: [(33 * 256, 4, 0)] * 100000, 64),
    "tensors-11k": ("300,000 tensors of 11 KiB: every tile touches 3-4 tensors",
                    lambda: [(11 * 256, 4, 0)] * 300000, 64),
    "tensors-5k": ("200,000 tensors of 5 KiB: every tile on the general path",
                   lambda: [(5 * 256, 4, 0)] * 200000, 64),
    "tensors-5k-ragged": ("200,000 bf16 tensors of 5 KiB + 2 bytes: general path, every boundary "
                          "inside a lane's 16 bytes", lambda: [(5 * 512 + 1, 2, 0)] * 200000, 64),
}


def config_layout_variant(name, device="cpu"):
    _, build, max_gap = LAYOUT_VARIANTS[name]
    return fragmented_shard(build(), 4 * MiB, SEED_BASE + 3, device, name=name, max_gap=max_gap)


def config_llama70b(device):
    return param_shard("llama70b-dp64", llama70b_dp64_numels(), 8 * MiB, SEED_BASE + 5, device)


def corrupt_chunks(n_chunks, chunk_bytes, seed=SEED_BASE + 5, fraction=0.01):
    """Seeded choice of round(fraction*n_chunks) distinct chunks and one bit position in each:
    list of (chunk, byte offset in chunk, bit)."""
    rng = np.random.default_rng(seed)
    k = max(1, int(round(fraction * n_chunks)))
    chunks = np.sort(rng.choice(n_chunks, size=k, replace=False))
    return [(int(c), int(rng.integers(0, chunk_bytes)), int(rng.integers(0, 8))) for c in chunks]


# ---- host views -------------------------------------------------------------------------------

def to_numpy_bytes(t):
    """Raw bytes of a (CPU or device) tensor as a fresh contiguous numpy uint8 array."""
    t = t.detach().contiguous()
    return t.view(torch.uint8).cpu().numpy().copy() if t.dtype != torch.uint8 \
        else t.cpu().numpy().copy()


def numpy_alias(t):
    """Numpy array aliasing a CPU tensor's memory (bf16 comes back as uint16 bit patterns)."""
    assert t.device.type == "cpu"
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
