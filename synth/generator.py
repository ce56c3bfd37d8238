"""Seeded synthetic training-state inputs.

This module serves the tests, the benchmark and the smoke check.  It knows
nothing about parallelism configurations or resharding: a caller hands it a
generic description of a stored block of a tensor (`ShardDesc`: which box of the
full tensor, stored in which axis order, at which byte offset) and it writes
values that are a pure function of (seed, tensor id, state kind, position in
the full tensor).  Because every value is addressable in O(1), the same
function yields both the source shards of a job and, independently, the
contents any re-partitioned shard must have.

All arithmetic is either integer (wrapping int64) or a single IEEE fp32
multiply of an exactly representable integer, so CPU and GPU results are
bit-identical.

Value streams (the paper's jobs are GPT-3 models trained with Adam; their
weights are not available, so these stand in for them):
  "u11"   fp32, uniform on [-1, 1)                     (tiny config weights)
  "n02"   fp32, bell-shaped (sum of four 16-bit uniforms), mean 0, std 0.02
  "bf16w" bf16, round-to-nearest-even of the "n02" value of the same element
  "m"     fp32, bell-shaped, std 1e-3                  (Adam first moment)
  "v"     fp32, uniform on [0, 1e-6)                   (Adam second moment)
  "index" any width: low bits of a mix of the element's linear index, for
          exact misplacement detection
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Iterable, Sequence

import numpy as np
import torch

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def _s64(x: int) -> int:
    """Python int -> the signed 64-bit integer with the same low 64 bits."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix_py(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 lanes."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    return z ^ _lsr(z, 31)


def stream_key(seed: int, tensor_id: int, stream: int) -> int:
    """64-bit key of one (seed, tensor, stream) value stream."""
    k = _mix_py(seed * 0xD6E8FEB86659FD93 + 0x1234567)
    k = _mix_py(k ^ (tensor_id * 0xA0761D6478BD642F + 0x51))
    k = _mix_py(k ^ (stream * 0xE7037ED1A0B428DB + 0x77))
    return k


def hash64(key: int, lin: torch.Tensor) -> torch.Tensor:
    """Counter-based hash: element `lin` of stream `key` -> 64 random bits (int64)."""
    return _mix((lin + 1) * _s64(_GOLDEN) + _s64(key))


# ---------------------------------------------------------------------------
# state mixes: per state kind (element bytes, value stream name)
# ---------------------------------------------------------------------------
MIX_TINY = ((4, "u11"), (4, "m"), (4, "v"))                # fp32 w, m, v: 12 B/param
MIX_GPT = ((2, "bf16w"), (4, "n02"), (4, "m"), (4, "v"))   # bf16 w + fp32 master, m, v: 14 B/param
MIX_INDEX_TINY = ((4, "index"), (4, "index"), (4, "index"))
MIX_INDEX_GPT = ((2, "index"), (4, "index"), (4, "index"), (4, "index"))

_SUM4_MEAN = 2 * 65535
_SUM4_STD = 65536.0 * math.sqrt(4.0 / 12.0)


def _sum4(h: torch.Tensor) -> torch.Tensor:
    return ((h & 0xFFFF) + (_lsr(h, 16) & 0xFFFF) + (_lsr(h, 32) & 0xFFFF) + _lsr(h, 48)) - _SUM4_MEAN


def values(seed: int, tensor_id: int, kind: int, stream: str, elem_bytes: int,
           lin: torch.Tensor) -> torch.Tensor:
    """Values of elements with canonical linear indices `lin` (int64 tensor).

    Returns a tensor of the stream's dtype with lin's shape.  "bf16w" reads the
    stream of state kind `kind + 1` (its fp32 master copy) and rounds it.
    """
    if stream == "index":
        bits = lin + _s64(tensor_id * 0x9E3779B1 + kind * 0x85EBCA6B)
        if elem_bytes == 1:
            return ((bits & 0xFF) - ((bits & 0x80) << 1)).to(torch.int8)
        if elem_bytes == 2:
            return ((bits & 0xFFFF) - ((bits & 0x8000) << 1)).to(torch.int16)
        if elem_bytes == 4:
            return ((bits & 0xFFFFFFFF) - ((bits & 0x80000000) << 1)).to(torch.int32)
        if elem_bytes == 8:
            return bits
        raise ValueError("index stream: element bytes must be 1, 2, 4 or 8")
    if stream == "bf16w":
        return values(seed, tensor_id, kind + 1, "n02", 4, lin).to(torch.bfloat16)
    h = hash64(stream_key(seed, tensor_id, kind), lin)
    if stream == "u11":
        b = _lsr(h, 40) - (1 << 23)
        return b.to(torch.float32) * float(2.0 ** -23)
    if stream == "n02":
        return _sum4(h).to(torch.float32) * float(np.float32(0.02 / _SUM4_STD))
    if stream == "m":
        return _sum4(h).to(torch.float32) * float(np.float32(1e-3 / _SUM4_STD))
    if stream == "v":
        return _lsr(h, 40).to(torch.float32) * float(np.float32(1e-6 * 2.0 ** -24))
    raise ValueError(f"unknown value stream {stream!r}")


# ---------------------------------------------------------------------------
# stored blocks
# ---------------------------------------------------------------------------
@dataclass(frozen=True)
class ShardDesc:
    """One stored block of one state tensor inside a flat rank buffer.

    full_shape: shape of the whole (unpartitioned) tensor in its canonical axis order
    lo, hi:     per canonical axis, the half-open range this block covers
    perm:       storage order; stored axis i is canonical axis perm[i]; the block
                is dense row-major in that order
    """
    tensor_id: int
    kind: int
    elem_bytes: int
    offset: int
    full_shape: tuple
    lo: tuple
    hi: tuple
    perm: tuple

    @property
    def stored_shape(self) -> tuple:
        return tuple(self.hi[a] - self.lo[a] for a in self.perm)

    @property
    def numel(self) -> int:
        n = 1
        for a in range(len(self.full_shape)):
            n *= self.hi[a] - self.lo[a]
        return n

    @property
    def nbytes(self) -> int:
        return self.numel * self.elem_bytes


def canonical_strides(full_shape: Sequence[int]) -> tuple:
    """Row-major element strides of the canonical view; the extent of axis 0
    never enters, so tensors that differ only in (padded) leading extent share
    linear indices."""
    st = [1] * len(full_shape)
    for a in range(len(full_shape) - 2, -1, -1):
        st[a] = st[a + 1] * full_shape[a + 1]
    return tuple(st)


def linear_index(desc: ShardDesc, device, r0: int = 0, r1: int | None = None) -> torch.Tensor:
    """Canonical linear index of every element of stored rows [r0, r1) (stored
    axis 0) of the block, shaped like the stored block."""
    cs = canonical_strides(desc.full_shape)
    shp = desc.stored_shape
    if r1 is None:
        r1 = shp[0]
    nd = len(shp)
    total = torch.zeros((), dtype=torch.int64, device=device)
    for i, a in enumerate(desc.perm):
        start, stop = (r0, r1) if i == 0 else (0, shp[i])
        ar = (torch.arange(start, stop, dtype=torch.int64, device=device) + desc.lo[a]) * cs[a]
        view = [1] * nd
        view[i] = stop - start
        total = total + ar.view(view)
    return total


_CHUNK_ELEMS = 1 << 25


def _row_chunks(desc: ShardDesc):
    shp = desc.stored_shape
    if desc.numel == 0:
        return
    per_row = desc.numel // shp[0]
    step = max(1, _CHUNK_ELEMS // max(1, per_row))
    for r0 in range(0, shp[0], step):
        yield r0, min(shp[0], r0 + step), per_row


def block_values(seed: int, desc: ShardDesc, stream: str, device,
                 r0: int = 0, r1: int | None = None,
                 zero_from_row: int | None = None) -> torch.Tensor:
    """Values of stored rows [r0, r1) of a block.  Elements whose canonical
    axis-0 coordinate is >= zero_from_row are zero (rows that exist only as
    padding of the new layout)."""
    lin = linear_index(desc, device, r0, r1)
    val = values(seed, desc.tensor_id, desc.kind, stream, desc.elem_bytes, lin)
    if zero_from_row is not None:
        cs0 = canonical_strides(desc.full_shape)[0]
        val = torch.where(lin >= zero_from_row * cs0, torch.zeros((), dtype=val.dtype, device=device), val)
    return val


def fill_buffer(buf: torch.Tensor, descs: Iterable[ShardDesc], seed: int,
                mix: Sequence[tuple], zero_from_row=None) -> None:
    """Write every described block into the flat uint8 buffer `buf`.

    zero_from_row: optional callable desc -> row or None (see block_values)."""
    for d in descs:
        eb, stream = mix[d.kind]
        assert eb == d.elem_bytes
        z = zero_from_row(d) if zero_from_row is not None else None
        for r0, r1, per_row in _row_chunks(d):
            v = block_values(seed, d, stream, buf.device, r0, r1, z).contiguous()
            b0 = d.offset + r0 * per_row * eb
            buf[b0:b0 + (r1 - r0) * per_row * eb] = v.view(-1).view(torch.uint8)


def count_mismatch(buf: torch.Tensor, descs: Iterable[ShardDesc], seed: int,
                   mix: Sequence[tuple], zero_from_row=None) -> int:
    """Number of blocks of `buf` that differ from their closed-form contents."""
    bad = 0
    for d in descs:
        eb, stream = mix[d.kind]
        z = zero_from_row(d) if zero_from_row is not None else None
        ok = True
        for r0, r1, per_row in _row_chunks(d):
            v = block_values(seed, d, stream, buf.device, r0, r1, z).contiguous()
            b0 = d.offset + r0 * per_row * eb
            if not torch.equal(buf[b0:b0 + (r1 - r0) * per_row * eb], v.view(-1).view(torch.uint8)):
                ok = False
        bad += 0 if ok else 1
    return bad


# ---------------------------------------------------------------------------
# dataset state
# ---------------------------------------------------------------------------
def epoch_order(n_samples: int, seed: int) -> np.ndarray:
    """Global sample order of one epoch: a seeded permutation of 0..n-1 (uint64)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.permutation(n_samples).astype(np.uint64)
