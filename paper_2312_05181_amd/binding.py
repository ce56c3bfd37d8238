"""ctypes binding of libtpx: argument marshalling only.  Every step of the path runs
inside the library (host planner in C++, execution in HIP kernels); nothing here
computes, and there is no fallback: if the library cannot be loaded, importing
this module fails."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

# Device memory and streams come from PyTorch, so the process must use exactly one HIP runtime: the one
# PyTorch ships.  libtpx.so names the runtime by soname only; importing torch first makes the dynamic
# linker resolve it to the copy torch has already loaded.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtpx.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2312_05181_amd.build` "
                      "(there is no CPU fallback)")
_lib = C.CDLL(LIB_PATH)

TPX_OK = 0
TPX_ERR_INVALID_ARG, TPX_ERR_INDIVISIBLE, TPX_ERR_BAD_STAGE_MAP, TPX_ERR_OOM, TPX_ERR_HIP = -1, -2, -3, -4, -5
TPX_ERR_MISALIGNED, TPX_ERR_CURSOR, TPX_ERR_UNRECOVERABLE, TPX_ERR_STALE_WORKSPACE, TPX_ERR_TOO_LARGE = -6, -7, -8, -9, -10
TPX_OFFSET_AUTO = 2 ** 64 - 1
TPX_STATIC_WORKSPACE_BYTES = 4 << 20
TPX_MAX_RANKS = 128
SIDE_SRC, SIDE_DST = 0, 1
MODEL_TIED_HEAD = 1
BOX_COPY, BOX_FILL, BOX_TRANSPOSE = 0, 1, 2
TILE_COPY, TILE_FILL, TILE_TRANSPOSE, TILE_GATHER, TILE_MERGE, TILE_PACK = 0, 1, 2, 3, 4, 5


class TpxError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"tpx status {status}: {message}")
        self.status = status


class tpx_model(C.Structure):
    _fields_ = [("n_layers", C.c_uint32), ("hidden", C.c_uint32), ("n_heads", C.c_uint32), ("ffn", C.c_uint32),
                ("vocab_true", C.c_uint32), ("max_pos", C.c_uint32), ("vocab_divisor", C.c_uint32),
                ("n_state_kinds", C.c_uint32), ("state_elem_bytes", C.c_uint8 * 4), ("flags", C.c_uint32)]


class tpx_parallel(C.Structure):
    _fields_ = [("T", C.c_uint32), ("P", C.c_uint32), ("D", C.c_uint32),
                ("stage_first_layer", C.POINTER(C.c_uint32)), ("qkv_layout", C.c_uint32),
                ("w_transposed", C.c_uint32), ("rank_alive", C.POINTER(C.c_uint8)), ("layer_stage", C.POINTER(C.c_uint32)),
                ("shard_kinds", C.c_uint32)]


class tpx_entry(C.Structure):
    _fields_ = [("tensor_id", C.c_uint32), ("kind", C.c_uint32), ("elem_bytes", C.c_uint32), ("ndim", C.c_uint32),
                ("name", C.c_uint32), ("layer", C.c_int32), ("offset", C.c_uint64), ("nbytes", C.c_uint64),
                ("full_shape", C.c_uint64 * 4), ("lo", C.c_uint64 * 4), ("hi", C.c_uint64 * 4),
                ("perm", C.c_uint32 * 4)]


class tpx_box(C.Structure):
    _fields_ = [("kind", C.c_uint32), ("src_rank", C.c_uint32), ("dst_rank", C.c_uint32), ("n_dst", C.c_uint32),
                ("dst_rank_stride", C.c_uint32), ("ndim", C.c_uint32),
                ("elem_bytes", C.c_uint32), ("tensor_id", C.c_uint32), ("src_off", C.c_uint64),
                ("dst_off", C.c_uint64), ("run_bytes", C.c_uint64), ("extent", C.c_uint64 * 4),
                ("src_stride", C.c_uint64 * 4), ("dst_stride", C.c_uint64 * 4)]


class tpx_tile(C.Structure):
    _fields_ = [("src_off", C.c_uint64), ("dst_off", C.c_uint64), ("src_pitch", C.c_uint64),
                ("dst_pitch", C.c_uint64), ("src_step", C.c_uint64), ("dst_step", C.c_uint64),
                ("run_units", C.c_uint32), ("nrows", C.c_uint32), ("src_rank", C.c_uint16),
                ("dst_rank", C.c_uint16), ("kind", C.c_uint8), ("unit_log2", C.c_uint8), ("n_dst", C.c_uint8),
                ("dst_rank_stride", C.c_uint8), ("seg_first", C.c_uint32), ("n_seg", C.c_uint32),
                ("seg_units", C.c_uint32), ("pad_", C.c_uint32)]


class tpx_segment(C.Structure):
    _fields_ = [("src_off", C.c_uint64), ("src_pitch", C.c_uint64), ("src_rank", C.c_uint32), ("units", C.c_uint32),
                ("dst_off", C.c_uint64)]


class tpx_ptc(C.Structure):
    _fields_ = [("n_ranks", C.c_uint32), ("n_entries", C.POINTER(C.c_uint32)),
                ("entries", C.POINTER(C.POINTER(tpx_entry))), ("rank_bytes", C.POINTER(C.c_uint64)),
                ("rank_alive", C.POINTER(C.c_uint8))]


class tpx_plan_opts(C.Structure):
    _fields_ = [("tile_bytes", C.c_uint64), ("max_multicast", C.c_uint32), ("share_reads", C.c_uint32),
                ("pack_bytes", C.c_uint32), ("reserved_", C.c_uint32)]


class tpx_query(C.Structure):
    _fields_ = [("tensor_id", C.c_uint32), ("kind", C.c_uint32), ("lo", C.c_uint64 * 4), ("hi", C.c_uint64 * 4)]


class tpx_stats_t(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("n_pieces", "n_boxes", "n_tiles", "bytes_read", "bytes_written",
                                          "bytes_fill", "bytes_cross_rank", "plan_ns")]


assert C.sizeof(tpx_tile) == 80

_P = C.c_void_p
_sigs = {
    "tpx_plan": (C.c_int, [C.POINTER(tpx_model), C.POINTER(tpx_parallel), C.POINTER(tpx_parallel),
                           C.POINTER(tpx_plan_opts), C.POINTER(_P)]),
    "tpx_plan_ptc": (C.c_int, [C.POINTER(tpx_ptc), C.POINTER(tpx_ptc), C.POINTER(tpx_plan_opts), C.POINTER(_P)]),
    "tpx_plan_query": (C.c_int, [C.POINTER(tpx_ptc), C.c_uint32, C.POINTER(tpx_query), C.POINTER(tpx_plan_opts),
                                 C.POINTER(_P)]),
    "tpx_plan_dataset": (C.c_int, [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32,
                                   C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(tpx_plan_opts),
                                   C.POINTER(_P)]),
    "tpx_num_buffers": (C.c_uint32, [_P, C.c_int]),
    "tpx_buffer_bytes": (C.c_uint64, [_P, C.c_int, C.c_uint32]),
    "tpx_num_entries": (C.c_uint32, [_P, C.c_int, C.c_uint32]),
    "tpx_manifest": (C.c_int, [_P, C.c_int, C.c_uint32, C.c_uint32, C.POINTER(tpx_entry)]),
    "tpx_param_name": (C.c_char_p, [C.c_uint32]),
    "tpx_stats": (C.c_int, [_P, C.POINTER(tpx_stats_t)]),
    "tpx_num_boxes": (C.c_uint64, [_P]),
    "tpx_get_box": (C.c_int, [_P, C.c_uint64, C.POINTER(tpx_box)]),
    "tpx_num_tiles": (C.c_uint64, [_P]),
    "tpx_get_tile": (C.c_int, [_P, C.c_uint64, C.POINTER(tpx_tile)]),
    "tpx_num_segments": (C.c_uint64, [_P]),
    "tpx_get_segment": (C.c_int, [_P, C.c_uint64, C.POINTER(tpx_segment)]),
    "tpx_traffic": (C.c_int, [_P, C.POINTER(C.c_uint64)]),
    "tpx_workspace_bytes": (C.c_uint64, [_P]),
    "tpx_execute": (C.c_int, [_P, C.POINTER(_P), C.POINTER(_P), _P, _P]),
    "tpx_execute_static": (C.c_int, [_P, C.POINTER(_P), C.POINTER(_P), _P]),
    "tpx_prepare": (C.c_int, [_P, _P, _P]),
    "tpx_workspace_forget": (None, [_P]),
    "tpx_workspace_check": (C.c_int, [_P, _P, _P]),
    "tpx_free": (None, [_P]),
    "tpx_last_error": (C.c_char_p, []),
    "tpx_set_option": (C.c_int, [C.c_char_p, C.c_uint64]),
    "tpx_probe_copy": (C.c_int, [_P, _P, C.c_uint64, _P]),
    "tpx_probe_read": (C.c_int, [_P, C.c_uint64, _P, _P]),
    "tpx_probe_fill": (C.c_int, [_P, C.c_uint64, C.c_uint32, _P]),
}
for _name, (_res, _args) in _sigs.items():
    _f = getattr(_lib, _name)
    _f.restype = _res
    _f.argtypes = _args
EXPORTS = tuple(_sigs)


def _check(st: int) -> None:
    if st != TPX_OK:
        raise TpxError(st, _lib.tpx_last_error().decode())


def _model_struct(n_layers, hidden, n_heads, ffn, vocab_true, max_pos=1024, vocab_divisor=0,
                  state_elem_bytes=(2, 4, 4, 4), tied_head=False) -> tpx_model:
    m = tpx_model(n_layers, hidden, n_heads, ffn, vocab_true, max_pos, vocab_divisor, len(state_elem_bytes))
    for i, b in enumerate(state_elem_bytes):
        m.state_elem_bytes[i] = b
    m.flags = MODEL_TIED_HEAD if tied_head else 0
    return m


def _opts_struct(opts) -> "C.POINTER(tpx_plan_opts)":
    """opts: None or a dict with any of tile_bytes, max_multicast, share_reads, pack_bytes."""
    if not opts:
        return None
    unknown = set(opts) - {"tile_bytes", "max_multicast", "share_reads", "pack_bytes"}
    if unknown:
        raise TpxError(TPX_ERR_INVALID_ARG, f"unknown plan option {sorted(unknown)[0]}")
    return C.pointer(tpx_plan_opts(int(opts.get("tile_bytes", 0)), int(opts.get("max_multicast", 0)),
                                   int(opts.get("share_reads", 0)), int(opts.get("pack_bytes", 0)), 0))


def _parallel_struct(T, P, D, stage_first_layer=None, qkv_layout=0, w_transposed=0, rank_alive=None, shard_kinds=0,
                     layer_stage=None, n_layers=None):
    # the library reads exactly P+1 / n_layers / T*P*D elements behind these pointers: refuse shorter or longer lists here
    if stage_first_layer is not None and len(stage_first_layer) != P + 1:
        raise TpxError(TPX_ERR_INVALID_ARG, f"stage_first_layer needs P+1 = {P + 1} entries, got {len(stage_first_layer)}")
    if rank_alive is not None and len(rank_alive) != T * P * D:
        raise TpxError(TPX_ERR_INVALID_ARG, f"rank_alive needs T*P*D = {T * P * D} entries, got {len(rank_alive)}")
    if layer_stage is not None and n_layers is not None and len(layer_stage) != n_layers:
        raise TpxError(TPX_ERR_INVALID_ARG, f"layer_stage needs one entry per layer ({n_layers}), got {len(layer_stage)}")
    keep = []
    p = tpx_parallel(T, P, D)
    if stage_first_layer is not None:
        arr = (C.c_uint32 * len(stage_first_layer))(*stage_first_layer)
        keep.append(arr)
        p.stage_first_layer = C.cast(arr, C.POINTER(C.c_uint32))
    p.qkv_layout, p.w_transposed, p.shard_kinds = qkv_layout, w_transposed, shard_kinds
    if rank_alive is not None:
        arr = (C.c_uint8 * len(rank_alive))(*[1 if a else 0 for a in rank_alive])
        keep.append(arr)
        p.rank_alive = C.cast(arr, C.POINTER(C.c_uint8))
    if layer_stage is not None:
        arr = (C.c_uint32 * len(layer_stage))(*layer_stage)
        keep.append(arr)
        p.layer_stage = C.cast(arr, C.POINTER(C.c_uint32))
    return p, keep


class Plan:
    """Owner of one tpx_plan_t handle."""

    def __init__(self, handle: int, dst_cursors: Optional[list] = None):
        self._h = _P(handle)
        self.dst_cursors = dst_cursors

    def close(self, _free=_lib.tpx_free) -> None:
        # _free is bound at definition time: at interpreter shutdown the module globals may be gone already
        if self._h:
            _free(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def num_buffers(self, side: int) -> int:
        return _lib.tpx_num_buffers(self._h, side)

    def buffer_bytes(self, side: int, rank: int) -> int:
        return _lib.tpx_buffer_bytes(self._h, side, rank)

    def manifest(self, side: int, rank: int) -> list:
        out = []
        for i in range(_lib.tpx_num_entries(self._h, side, rank)):
            e = tpx_entry()
            _check(_lib.tpx_manifest(self._h, side, rank, i, C.byref(e)))
            out.append(e)
        return out

    def stats(self) -> dict:
        s = tpx_stats_t()
        _check(_lib.tpx_stats(self._h, C.byref(s)))
        return {n: getattr(s, n) for n, _ in tpx_stats_t._fields_}

    def boxes(self) -> list:
        out = []
        for i in range(_lib.tpx_num_boxes(self._h)):
            b = tpx_box()
            _check(_lib.tpx_get_box(self._h, i, C.byref(b)))
            out.append(b)
        return out

    def num_tiles(self) -> int:
        return _lib.tpx_num_tiles(self._h)

    def tiles(self) -> list:
        out = []
        for i in range(_lib.tpx_num_tiles(self._h)):
            t = tpx_tile()
            _check(_lib.tpx_get_tile(self._h, i, C.byref(t)))
            out.append(t)
        return out

    def segments(self) -> list:
        out = []
        for i in range(_lib.tpx_num_segments(self._h)):
            g = tpx_segment()
            _check(_lib.tpx_get_segment(self._h, i, C.byref(g)))
            out.append(g)
        return out

    def traffic(self) -> list:
        """[source rank][destination rank] -> bytes moved between the two buffers."""
        ns, nd = self.num_buffers(SIDE_SRC), self.num_buffers(SIDE_DST)
        out = (C.c_uint64 * max(1, ns * nd))()
        _check(_lib.tpx_traffic(self._h, out))
        return [[out[i * nd + j] for j in range(nd)] for i in range(ns)]

    def workspace_bytes(self) -> int:
        return _lib.tpx_workspace_bytes(self._h)

    def execute(self, src_ptrs: Sequence[int], dst_ptrs: Sequence[int], workspace_ptr: int, stream: int = 0) -> None:
        """Launch the reshard. All pointers are device addresses (ints); stream is a hipStream_t (int)."""
        src = (_P * max(1, len(src_ptrs)))(*[_P(p) for p in src_ptrs])
        dst = (_P * max(1, len(dst_ptrs)))(*[_P(p) for p in dst_ptrs])
        if len(src_ptrs) != self.num_buffers(SIDE_SRC) or len(dst_ptrs) != self.num_buffers(SIDE_DST):
            raise TpxError(TPX_ERR_INVALID_ARG, "one pointer per rank buffer is required")
        _check(_lib.tpx_execute(self._h, src, dst, _P(workspace_ptr), _P(stream)))

    def execute_static(self, src_ptrs: Sequence[int], dst_ptrs: Sequence[int], stream: int = 0) -> None:
        """The same launch with the plan tables in the library's static device array: nothing is allocated."""
        if len(src_ptrs) != self.num_buffers(SIDE_SRC) or len(dst_ptrs) != self.num_buffers(SIDE_DST):
            raise TpxError(TPX_ERR_INVALID_ARG, "one pointer per rank buffer is required")
        src = (_P * max(1, len(src_ptrs)))(*[_P(p) for p in src_ptrs])
        dst = (_P * max(1, len(dst_ptrs)))(*[_P(p) for p in dst_ptrs])
        _check(_lib.tpx_execute_static(self._h, src, dst, _P(stream)))

    def prepare(self, workspace_ptr: int, stream: int = 0) -> None:
        _check(_lib.tpx_prepare(self._h, _P(workspace_ptr), _P(stream)))

    def workspace_check(self, workspace_ptr: int, stream: int = 0) -> None:
        """Wait for the stream and raise TpxError(TPX_ERR_STALE_WORKSPACE) unless the workspace holds this plan."""
        _check(_lib.tpx_workspace_check(self._h, _P(workspace_ptr), _P(stream)))


def tpx_plan(model: dict, src: dict, dst: dict, opts: Optional[dict] = None) -> Plan:
    """model: kwargs of the GPT-style model; src / dst: kwargs T, P, D[, stage_first_layer, qkv_layout,
    w_transposed, rank_alive, shard_kinds, layer_stage (one stage index per layer)]; opts: tile_bytes,
    max_multicast, share_reads of this plan."""
    m = _model_struct(**model)
    s, keep_s = _parallel_struct(n_layers=m.n_layers, **src)
    d, keep_d = _parallel_struct(n_layers=m.n_layers, **dst)
    h = _P()
    _check(_lib.tpx_plan(C.byref(m), C.byref(s), C.byref(d), _opts_struct(opts), C.byref(h)))
    del keep_s, keep_d
    return Plan(h.value)


def _ptc_struct(manifests, rank_bytes=None, rank_alive=None):
    """manifests: per rank, a list of objects with attributes tensor_id, kind, elem_bytes, offset, full_shape,
    lo, hi, perm (synth.ShardDesc has them; name and layer are optional; offset None = TPX_OFFSET_AUTO)."""
    keep = []
    n = len(manifests)
    if rank_bytes is not None and len(rank_bytes) != n:
        raise TpxError(TPX_ERR_INVALID_ARG, f"rank_bytes needs one entry per rank ({n}), got {len(rank_bytes)}")
    if rank_alive is not None and len(rank_alive) != n:
        raise TpxError(TPX_ERR_INVALID_ARG, f"rank_alive needs one entry per rank ({n}), got {len(rank_alive)}")
    counts = (C.c_uint32 * max(1, n))(*[len(m) for m in manifests])
    ptrs = (C.POINTER(tpx_entry) * max(1, n))()
    for r, man in enumerate(manifests):
        arr = (tpx_entry * max(1, len(man)))()
        for i, d in enumerate(man):
            e = arr[i]
            e.tensor_id, e.kind, e.elem_bytes = d.tensor_id, d.kind, d.elem_bytes
            e.offset = TPX_OFFSET_AUTO if d.offset is None else d.offset
            e.ndim = len(d.full_shape)
            if not (len(d.lo) == len(d.hi) == len(d.perm) == e.ndim <= 4):
                raise TpxError(TPX_ERR_INVALID_ARG, "lo, hi, perm and full_shape must have the same length, at most 4")
            e.name, e.layer = getattr(d, "name", 0), getattr(d, "layer", -1)
            for k in range(e.ndim):
                e.full_shape[k], e.lo[k], e.hi[k], e.perm[k] = d.full_shape[k], d.lo[k], d.hi[k], d.perm[k]
        keep.append(arr)
        ptrs[r] = C.cast(arr, C.POINTER(tpx_entry))
    c = tpx_ptc(n, C.cast(counts, C.POINTER(C.c_uint32)), C.cast(ptrs, C.POINTER(C.POINTER(tpx_entry))))
    keep += [counts, ptrs]
    if rank_bytes is not None:
        rb = (C.c_uint64 * max(1, n))(*rank_bytes)
        keep.append(rb)
        c.rank_bytes = C.cast(rb, C.POINTER(C.c_uint64))
    if rank_alive is not None:
        ra = (C.c_uint8 * max(1, n))(*[1 if a else 0 for a in rank_alive])
        keep.append(ra)
        c.rank_alive = C.cast(ra, C.POINTER(C.c_uint8))
    return c, keep


def tpx_plan_ptc(src_manifests, dst_manifests, src_bytes=None, dst_bytes=None, src_alive=None, dst_alive=None,
                 opts: Optional[dict] = None) -> Plan:
    """Plan between two explicitly given collections (any sharding expressible as boxes of tensors).
    src_alive: 0 = that source rank is lost; dst_alive: 0 = that destination rank is not to be built."""
    s, keep_s = _ptc_struct(src_manifests, src_bytes, src_alive)
    d, keep_d = _ptc_struct(dst_manifests, dst_bytes, dst_alive)
    h = _P()
    _check(_lib.tpx_plan_ptc(C.byref(s), C.byref(d), _opts_struct(opts), C.byref(h)))
    del keep_s, keep_d
    return Plan(h.value)


def tpx_plan_query(src_manifests, queries, src_bytes=None, src_alive=None, opts: Optional[dict] = None) -> Plan:
    """Range queries on a stored collection (paper section 5.2: "/2/embedding/weight[:, 2:4]"): queries is a list of
    (tensor_id, kind, lo, hi) boxes in the full tensors' coordinates; the plan gathers them, from whichever ranks
    hold the pieces, into ONE destination buffer laid out by the library (plan.manifest(1, 0) gives the offsets,
    plan.buffer_bytes(1, 0) the size)."""
    s, keep_s = _ptc_struct(src_manifests, src_bytes, src_alive)
    qs = (tpx_query * max(1, len(queries)))()
    for q, (tensor_id, kind, lo, hi) in zip(qs, queries):
        if not (len(lo) == len(hi) <= 4):
            raise TpxError(TPX_ERR_INVALID_ARG, "a query's lo and hi must have the same length, at most 4")
        q.tensor_id, q.kind = tensor_id, kind
        for k in range(len(lo)):
            q.lo[k], q.hi[k] = lo[k], hi[k]
    h = _P()
    _check(_lib.tpx_plan_query(C.byref(s), len(queries), qs, _opts_struct(opts), C.byref(h)))
    del keep_s
    return Plan(h.value)


def tpx_plan_dataset(n_samples: int, global_batch: int, D_src: int, D_dst: int, src_cursors: Sequence[int],
                     index_elem_bytes: int = 8, opts: Optional[dict] = None) -> Plan:
    if len(src_cursors) != D_src:
        raise TpxError(TPX_ERR_INVALID_ARG, "one cursor per source replica is required")
    cur = (C.c_uint64 * max(1, D_src))(*src_cursors)
    out = (C.c_uint64 * max(1, D_dst))()
    h = _P()
    _check(_lib.tpx_plan_dataset(n_samples, global_batch, index_elem_bytes, D_src, D_dst, cur, out, _opts_struct(opts),
                                 C.byref(h)))
    return Plan(h.value, [int(out[i]) for i in range(D_dst)])


def tpx_execute(plan: Plan, src_ptrs, dst_ptrs, workspace_ptr, stream=0) -> None:
    plan.execute(src_ptrs, dst_ptrs, workspace_ptr, stream)


def tpx_execute_static(plan: Plan, src_ptrs, dst_ptrs, stream=0) -> None:
    plan.execute_static(src_ptrs, dst_ptrs, stream)


def tpx_free(plan: Plan) -> None:
    plan.close()


def tpx_workspace_forget(workspace_ptr: int = 0) -> None:
    """Tell the library that a workspace was overwritten or freed (0: all of them)."""
    _lib.tpx_workspace_forget(_P(workspace_ptr))


def tpx_set_option(key: str, value: int) -> None:
    _check(_lib.tpx_set_option(key.encode(), value))


def tpx_probe_copy(dst_ptr: int, src_ptr: int, nbytes: int, stream: int = 0) -> None:
    _check(_lib.tpx_probe_copy(_P(dst_ptr), _P(src_ptr), nbytes, _P(stream)))


def tpx_probe_read(src_ptr: int, nbytes: int, sink_ptr: int, stream: int = 0) -> None:
    _check(_lib.tpx_probe_read(_P(src_ptr), nbytes, _P(sink_ptr), _P(stream)))


def tpx_probe_fill(dst_ptr: int, nbytes: int, value: int, stream: int = 0) -> None:
    _check(_lib.tpx_probe_fill(_P(dst_ptr), nbytes, value, _P(stream)))


def tpx_param_name(name: int) -> Optional[str]:
    s = _lib.tpx_param_name(name)
    return s.decode() if s else None
