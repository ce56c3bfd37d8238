"""Dataset-state planner (host side) against the dataset oracle, with the plan interpreted on the CPU."""
import numpy as np
import pytest

import paper_2312_05181_amd as tpx
import paper_2312_05181_amd.binding as B
import synth
from oracle import dataset as ods
from tests import helpers as H
from tests import host_exec


def _run(n, Bsz, D, D2, s, eb=8, how="boxes"):
    G = synth.epoch_order(n, 3) if n else np.zeros(0, dtype=np.uint64)
    if eb == 16:       # (offset, length) pairs: two 64-bit words per sample
        G = np.stack([G, G * np.uint64(7) + np.uint64(1)], axis=1)
    parts = ods.partition(G, Bsz, D)
    cur = ods.cursors_after(n, Bsz, D, s)
    want_parts, want_cur = ods.repartition(parts, cur, Bsz, D2)
    plan = tpx.tpx_plan_dataset(n, Bsz, D, D2, cur, index_elem_bytes=eb, opts=dict(tile_bytes=4096))
    assert plan.dst_cursors == want_cur
    assert [plan.buffer_bytes(0, j) for j in range(D)] == [p.nbytes for p in parts]
    assert [plan.buffer_bytes(1, j) for j in range(D2)] == [p.nbytes for p in want_parts]
    src = [np.ascontiguousarray(p).reshape(-1).view(np.uint8) for p in parts]
    got = [np.full(p.nbytes, H.POISON, dtype=np.uint8) for p in want_parts]
    cover = [np.zeros(len(g), dtype=np.int32) for g in got]
    (host_exec.run_boxes if how == "boxes" else host_exec.run_tiles)(plan, src, got, cover)
    for j in range(D2):
        assert np.array_equal(got[j], np.ascontiguousarray(want_parts[j]).reshape(-1).view(np.uint8)), j
        assert (cover[j] == 1).all()
    return plan


@pytest.mark.parametrize("how", ["boxes", "tiles"])
@pytest.mark.parametrize("n,Bsz,D,D2,s", [(100, 24, 6, 4, 2), (101, 24, 4, 6, 3), (53, 12, 2, 3, 0), (53, 12, 3, 1, 5),
                                          (96, 24, 6, 4, 4), (7, 12, 6, 4, 1), (0, 12, 2, 3, 0), (4096, 768, 6, 4, 3),
                                          (768 * 5 + 256, 768, 6, 4, 2), (1000, 48, 6, 6, 7), (1000, 48, 1, 6, 7)])
def test_dataset_plan_matches_oracle(n, Bsz, D, D2, s, how):
    _run(n, Bsz, D, D2, s, how=how)


def test_offset_length_pairs():
    _run(1000, 48, 6, 4, 5, eb=16)


def test_same_degree_is_one_copy_per_partition():
    plan = _run(1000, 48, 6, 6, 7)
    bx = plan.boxes()
    assert len(bx) == 6 and all(b.ndim == 0 and b.src_rank == b.dst_rank for b in bx)


def test_six_to_four_has_gcd_structured_runs():
    """B = 768: 6 -> 4 replicas cuts the batch at multiples of 128 and 192, so runs are 64 or 128 samples."""
    plan = _run(768 * 4, 768, 6, 4, 1)
    assert plan.stats()["n_pieces"] == 6 + 4 - 2
    assert sorted({b.run_bytes for b in plan.boxes()}) == [64 * 8, 128 * 8]


def test_dataset_errors():
    def st(fn):
        with pytest.raises(tpx.TpxError) as ei:
            fn()
        return ei.value.status
    assert st(lambda: tpx.tpx_plan_dataset(100, 24, 4, 2, [6, 6, 6, 5])) == B.TPX_ERR_CURSOR
    assert st(lambda: tpx.tpx_plan_dataset(100, 24, 4, 2, [7, 7, 7, 7])) == B.TPX_ERR_CURSOR
    assert st(lambda: tpx.tpx_plan_dataset(100, 24, 4, 2, [99, 6, 6, 6])) == B.TPX_ERR_CURSOR
    assert st(lambda: tpx.tpx_plan_dataset(100, 25, 4, 2, [0, 0, 0, 0])) == B.TPX_ERR_INDIVISIBLE
    assert st(lambda: tpx.tpx_plan_dataset(100, 24, 4, 0, [0, 0, 0, 0])) == B.TPX_ERR_INVALID_ARG
    assert st(lambda: tpx.tpx_plan_dataset(100, 24, 4, 2, [0, 0, 0, 0], index_elem_bytes=4)) == B.TPX_ERR_INVALID_ARG
