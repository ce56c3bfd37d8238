"""TEST INFRASTRUCTURE ONLY - CPU oracle of the model-state transformation.

The method is pure data movement, so the oracle is the plain definition rather
than the paper's plan (section 4.2 describes split / re-partition / merge; their
net effect is what is written out here): for every state tensor, paste the
source shards into the full tensor, then cut the full tensor the way the new
configuration wants it and store each piece where the new rank buffer keeps it.
Nothing is intersected, coalesced or tiled here.

Reading taken where the paper is silent: the authoritative source copy of a
shard is data-parallel replica d = 0 (and tensor-parallel rank t = 0 for
replicated tensors); all other holders must be bit-identical, which is checked.
Rows that exist only because the new vocabulary padding is larger are zero.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import Callable, Iterable, Optional

import numpy as np

from . import spec
from .spec import Model, Parallel

_UINT = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}


def _stored_shape(e) -> tuple:
    return tuple(e.hi[a] - e.lo[a] for a in e.perm)


def _to_canonical(block: np.ndarray, perm: tuple) -> np.ndarray:
    """stored block (axes in storage order) -> same block with canonical axis order."""
    inv = np.argsort(perm)
    return block.transpose(tuple(int(i) for i in inv))


def _to_stored(block: np.ndarray, perm: tuple) -> np.ndarray:
    return np.ascontiguousarray(block.transpose(perm))


def _box(lo, hi) -> tuple:
    return tuple(slice(l, u) for l, u in zip(lo, hi))


class Layout:
    """All rank manifests of one configuration, indexed by (tensor id, kind).

    Built either from a (model, parallel configuration) pair or from explicit manifests: a list, per rank,
    of (entries, buffer bytes) - the general form of a parallelizable tensor collection (paper section 4.1)."""

    def __init__(self, model: Optional[Model] = None, par: Optional[Parallel] = None, manifests=None):
        if manifests is None:
            manifests = [spec.rank_manifest(model, par, rank) for rank in range(par.n_ranks)]
        self.sizes = []
        self.by_tensor = {}
        for rank, (entries, nbytes) in enumerate(manifests):
            self.sizes.append(nbytes)
            for e in entries:
                self.by_tensor.setdefault((e.tensor_id, e.kind), []).append((rank, e))


def full_tensor(model: Model, par: Parallel, lay: Layout, tid: int, kind: int,
                read: Callable[[int, int, int], np.ndarray]) -> np.ndarray:
    """Reassemble one full state tensor (canonical axis order) from the shards of `par`.

    read(rank, offset, nbytes) returns that byte range of a source rank buffer."""
    hold = lay.by_tensor[(tid, kind)]
    e0 = hold[0][1]
    dt = _UINT[e0.elem_bytes]
    full = np.empty(e0.full_shape, dtype=dt)
    written = np.zeros(e0.full_shape, dtype=bool) if full.size <= (1 << 22) else None
    seen = {}
    for rank, e in hold:
        raw = read(rank, e.offset, _numel(e) * e.elem_bytes)
        block = _to_canonical(np.frombuffer(raw, dtype=dt).reshape(_stored_shape(e)), e.perm)
        key = (e.lo, e.hi)
        if key in seen:
            # replicas (data-parallel copies, replicated tensors, tied copies) must agree
            if not np.array_equal(seen[key], block):
                raise AssertionError(f"source replicas of tensor {tid} kind {kind} differ (rank {rank})")
            continue
        seen[key] = block
        full[_box(e.lo, e.hi)] = block
        if written is not None:
            written[_box(e.lo, e.hi)] = True
    if written is not None and not written.all():
        raise AssertionError(f"source shards of tensor {tid} do not cover it")
    if sum(b.size for b in seen.values()) != full.size:
        raise AssertionError(f"source shards of tensor {tid} do not tile it")
    return full


def _numel(e) -> int:
    n = 1
    for l, u in zip(e.lo, e.hi):
        n *= u - l
    return n


def reshard_tensor(model: Model, src: Parallel, dst: Parallel, src_lay: Layout, dst_lay: Layout,
                   tid: int, kind: int, read) -> list:
    """[(dst rank, entry, stored block)] for every destination holder of one state tensor."""
    full = full_tensor(model, src, src_lay, tid, kind, read)
    out = []
    for rank, e in dst_lay.by_tensor[(tid, kind)]:
        if e.full_shape != full.shape:
            # only the padded vocabulary extent (axis 0) may differ between configurations
            assert e.full_shape[1:] == full.shape[1:]
            grown = np.zeros(e.full_shape, dtype=full.dtype)
            n = min(e.full_shape[0], full.shape[0])
            grown[:n] = full[:n]
            use = grown
        else:
            use = full
        out.append((rank, e, _to_stored(use[_box(e.lo, e.hi)], e.perm)))
    return out


def reshard(model: Model, src: Parallel, dst: Parallel, src_bufs: list,
            tensor_ids: Optional[Iterable[int]] = None, threads: int = 1) -> list:
    """Destination rank buffers (uint8 arrays, POISON in every byte no tensor covers).

    src_bufs: one flat uint8 array per source rank.  tensor_ids restricts the
    work to some parameter tensors (all state kinds); other bytes stay POISON."""
    spec.check(model, src)
    spec.check(model, dst)
    src_lay, dst_lay = Layout(model, src), Layout(model, dst)
    if len(src_bufs) != src.n_ranks:
        raise ValueError("need one source buffer per source rank")
    for b, n in zip(src_bufs, src_lay.sizes):
        if b.nbytes != n:
            raise ValueError("source buffer size does not match its manifest")
    dst_bufs = [np.full(n, spec.POISON, dtype=np.uint8) for n in dst_lay.sizes]

    def read(rank, off, n):
        return src_bufs[rank][off:off + n]

    ids = range(model.n_tensors) if tensor_ids is None else list(tensor_ids)
    work = [(tid, kind) for tid in ids for kind in range(len(model.state_elem_bytes))]

    def one(tk):
        for rank, e, block in reshard_tensor(model, src, dst, src_lay, dst_lay, tk[0], tk[1], read):
            dst_bufs[rank][e.offset:e.offset + block.nbytes] = block.reshape(-1).view(np.uint8)

    if threads > 1:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(one, work))
    else:
        for tk in work:
            one(tk)
    return dst_bufs


def reshard_ptc(src_manifests, dst_manifests, src_bufs: list, threads: int = 1) -> list:
    """The same definition for collections given explicitly (expert, sequence, sharded-optimizer layouts ...):
    manifests are lists, per rank, of (entries, buffer bytes)."""
    src_lay, dst_lay = Layout(manifests=src_manifests), Layout(manifests=dst_manifests)
    if len(src_bufs) != len(src_lay.sizes):
        raise ValueError("need one source buffer per source rank")
    dst_bufs = [np.full(n, spec.POISON, dtype=np.uint8) for n in dst_lay.sizes]

    def read(rank, off, n):
        return src_bufs[rank][off:off + n]

    def one(tk):
        for rank, e, block in reshard_tensor(None, None, None, src_lay, dst_lay, tk[0], tk[1], read):
            dst_bufs[rank][e.offset:e.offset + block.nbytes] = block.reshape(-1).view(np.uint8)

    work = sorted(dst_lay.by_tensor)
    if threads > 1:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(one, work))
    else:
        for tk in work:
            one(tk)
    return dst_bufs


def state_bytes(model: Model, par: Parallel) -> int:
    """Total bytes of all rank buffers' tensors (without alignment gaps)."""
    total = 0
    for rank in range(par.n_ranks):
        entries, _ = spec.rank_manifest(model, par, rank)
        total += sum(_numel(e) * e.elem_bytes for e in entries)
    return total
