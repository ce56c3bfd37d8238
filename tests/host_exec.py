"""Test-side interpreters of a plan's public description (boxes and tiles), in numpy.
They let the CPU tests check the host planner against the oracle without a GPU.
They are not a product path: the library itself only ever executes plans with its HIP kernels."""
from __future__ import annotations

import numpy as np

import paper_2312_05181_amd.binding as B


def run_boxes(plan, src_bufs, dst_bufs, cover=None):
    """Apply every box to numpy uint8 buffers. cover (list of int arrays) counts writes per byte."""
    for b in plan.boxes():
        ext = [int(b.extent[k]) for k in range(b.ndim)]
        run = int(b.run_bytes)
        for idx in np.ndindex(*ext) if ext else [()]:
            so = int(b.src_off) + sum(i * int(b.src_stride[k]) for k, i in enumerate(idx))
            do = int(b.dst_off) + sum(i * int(b.dst_stride[k]) for k, i in enumerate(idx))
            for k in range(b.n_dst):
                r = b.dst_rank + k * b.dst_rank_stride
                if b.kind == B.BOX_FILL:
                    dst_bufs[r][do:do + run] = 0
                else:
                    dst_bufs[r][do:do + run] = src_bufs[b.src_rank][so:so + run]
                if cover is not None:
                    cover[r][do:do + run] += 1


def run_tiles(plan, src_bufs, dst_bufs, cover=None):
    """Apply every tile, unit by unit, exactly as the tile table defines it."""
    segs = plan.segments()
    for t in plan.tiles():
        unit = 1 << t.unit_log2
        if t.kind == B.TILE_MERGE:
            # whole destination rows; column block g of every row comes from segment seg_first + g
            row0 = int(t.src_off)
            widths = [segs[t.seg_first + g].units for g in range(t.n_seg)]
            assert sum(widths) == t.run_units and (t.seg_units == 0 or all(w == t.seg_units for w in widths))
            i = np.arange(t.nrows, dtype=np.int64)[:, None, None]
            kk = np.arange(unit, dtype=np.int64)[None, None, :]
            for c in range(t.n_dst):
                r = t.dst_rank + c * t.dst_rank_stride
                first = 0
                for g in range(t.n_seg):
                    sg = segs[t.seg_first + g]
                    j = np.arange(widths[g], dtype=np.int64)[None, :, None]
                    si = (int(sg.src_off) + (row0 + i) * int(sg.src_pitch) + j * unit + kk).reshape(-1)
                    di = (int(t.dst_off) + i * int(t.dst_pitch) + (first + j) * unit + kk).reshape(-1)
                    dst_bufs[r][di] = src_bufs[sg.src_rank][si]
                    if cover is not None:
                        np.add.at(cover[r], di, 1)
                    first += widths[g]
            continue
        if t.kind == B.TILE_PACK:
            # one row of units made of n_seg short moves, each with its own source and its own place in the destination
            assert t.nrows == 1 and unit == 16 and 1 <= t.n_seg <= 64
            first = 0
            for g in range(t.n_seg):
                sg = segs[t.seg_first + g]
                assert sg.src_pitch == first and sg.units > 0
                n = sg.units * 16
                for c in range(t.n_dst):
                    r = t.dst_rank + c * t.dst_rank_stride
                    dst_bufs[r][sg.dst_off:sg.dst_off + n] = src_bufs[sg.src_rank][sg.src_off:sg.src_off + n]
                    if cover is not None:
                        cover[r][sg.dst_off:sg.dst_off + n] += 1
                first += sg.units
            assert first == t.run_units
            continue
        i = np.arange(t.nrows, dtype=np.int64)[:, None, None]
        j = np.arange(t.run_units, dtype=np.int64)[None, :, None]
        k = np.arange(unit, dtype=np.int64)[None, None, :]
        di = (int(t.dst_off) + i * int(t.dst_pitch) + j * int(t.dst_step) + k).reshape(-1)
        for c in range(t.n_dst):
            r = t.dst_rank + c * t.dst_rank_stride
            if t.kind == B.TILE_FILL:
                dst_bufs[r][di] = 0
            else:
                si = (int(t.src_off) + i * int(t.src_pitch) + j * int(t.src_step) + k).reshape(-1)
                dst_bufs[r][di] = src_bufs[t.src_rank][si]
            if cover is not None:
                np.add.at(cover[r], di, 1)
