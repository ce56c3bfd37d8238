"""Host-side tests of libtpx (no GPU): exports, manifests against the oracle's layout, the plan
interpreted on the CPU against the oracle's output, closed forms of the plan, error codes."""
import math
import os
import re

import numpy as np
import pytest

import paper_2312_05181_amd as tpx
import paper_2312_05181_amd.binding as B
from oracle import reshard as oreshard
from oracle import spec
from oracle.spec import Model, Parallel
from tests import helpers as H
from tests import host_exec

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def mk(model: Model) -> dict:
    return dict(n_layers=model.n_layers, hidden=model.hidden, n_heads=model.n_heads, ffn=model.ffn,
                vocab_true=model.vocab_true, max_pos=model.max_pos, vocab_divisor=model.vocab_divisor,
                state_elem_bytes=tuple(model.state_elem_bytes), tied_head=model.tied_head)


def pk(par: Parallel, **extra) -> dict:
    d = dict(T=par.T, P=par.P, D=par.D, stage_first_layer=par.stage_first_layer, qkv_layout=par.qkv_layout,
             w_transposed=par.w_transposed, shard_kinds=par.shard_kinds, layer_stage=par.layer_stage)
    d.update(extra)
    return d


def plan_for(model, src, dst, dst_alive=None, opts=None, **kw):
    return tpx.tpx_plan(mk(model), pk(src, **kw), pk(dst, rank_alive=dst_alive) if dst_alive is not None else pk(dst), opts)


def test_library_exports_every_declared_symbol():
    import ctypes
    text = open(os.path.join(ROOT, "include", "tpx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(tpx_[a-z_]+)\s*\(", text))
    assert {"tpx_plan", "tpx_execute", "tpx_free"} <= declared
    lib = ctypes.CDLL(tpx.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(tpx.EXPORTS)


def _layout_cases():
    yield from ((H.CONFIGS[c][0], H.CONFIGS[c][1], H.CONFIGS[c][2]) for c in (1, 2, 3, 4, 5))
    yield H.GPT_1_3B, Parallel(4, 2, 2, shard_kinds=14), Parallel(2, 2, 4, shard_kinds=14, qkv_layout=1)   # sharded optimizer state
    yield H.TINY, Parallel(2, 1, 3, shard_kinds=7), Parallel(4, 2, 5, shard_kinds=2, w_transposed=1)
    yield H.GPT_1_3B, Parallel(2, 4, 1, layer_stage=tuple((l // 3) % 4 for l in range(24))), Parallel(4, 2, 1)     # 2 chunks of 3 layers per stage


@pytest.mark.parametrize("model,src,dst", list(_layout_cases()))
def test_manifest_equals_oracle_layout(model, src, dst):
    plan = plan_for(model, src, dst)
    for side, par in ((0, src), (1, dst)):
        assert plan.num_buffers(side) == par.n_ranks
        for r in range(par.n_ranks):
            entries, nbytes = spec.rank_manifest(model, par, r)
            assert plan.buffer_bytes(side, r) == nbytes
            got = plan.manifest(side, r)
            assert len(got) == len(entries)
            for g, e in zip(got, entries):
                nd = len(e.full_shape)
                assert (g.tensor_id, g.kind, g.elem_bytes, g.ndim, g.name, g.layer, g.offset) == \
                       (e.tensor_id, e.kind, e.elem_bytes, nd, e.name, e.layer, e.offset)
                assert tuple(g.full_shape[:nd]) == e.full_shape and tuple(g.lo[:nd]) == e.lo
                assert tuple(g.hi[:nd]) == e.hi and tuple(g.perm[:nd]) == e.perm
    assert tpx.tpx_param_name(4) == spec.NAMES[4][0] and tpx.tpx_param_name(16) is None


SMALL = Model(n_layers=4, hidden=24, n_heads=12, ffn=48, vocab_true=36, max_pos=5, state_elem_bytes=(4, 2))
SMALL_MIX = ((4, "u11"), (2, "index"))
ODD = Model(n_layers=2, hidden=12, n_heads=12, ffn=24, vocab_true=50, max_pos=3, vocab_divisor=4, state_elem_bytes=(2, 4))
ODD_MIX = ((2, "index"), (4, "u11"))
WIDE = Model(n_layers=2, hidden=128, n_heads=8, ffn=512, vocab_true=256, max_pos=16, state_elem_bytes=(2, 4, 4, 4),
             tied_head=True)

PAIRS = [
    (SMALL, SMALL_MIX, Parallel(2, 1, 1), Parallel(4, 2, 1)),
    (SMALL, SMALL_MIX, Parallel(4, 2, 1), Parallel(2, 4, 1)),
    (SMALL, SMALL_MIX, Parallel(4, 4, 2), Parallel(2, 4, 1, stage_first_layer=(0, 1, 1, 3, 4))),
    (SMALL, SMALL_MIX, Parallel(6, 1, 1), Parallel(1, 4, 1)),
    (SMALL, SMALL_MIX, Parallel(2, 2, 1), Parallel(2, 2, 2)),
    (SMALL, SMALL_MIX, Parallel(3, 1, 1), Parallel(3, 1, 1)),
    (SMALL, SMALL_MIX, Parallel(2, 1, 1, qkv_layout=1), Parallel(3, 2, 1)),
    (SMALL, SMALL_MIX, Parallel(2, 1, 1), Parallel(4, 1, 1, qkv_layout=1)),
    (SMALL, SMALL_MIX, Parallel(2, 1, 1), Parallel(3, 2, 1, w_transposed=1)),
    (SMALL, SMALL_MIX, Parallel(4, 1, 1, w_transposed=1, qkv_layout=1), Parallel(3, 1, 2)),
    (ODD, ODD_MIX, Parallel(3, 1, 1), Parallel(4, 1, 1)),
    (ODD, ODD_MIX, Parallel(4, 1, 1), Parallel(3, 1, 1)),
    (ODD, ODD_MIX, Parallel(3, 1, 1), Parallel(4, 2, 1, w_transposed=1)),
    (WIDE, H.synth.MIX_GPT, Parallel(2, 2, 1), Parallel(4, 1, 2)),
    (WIDE, H.synth.MIX_GPT, Parallel(8, 1, 1), Parallel(1, 2, 1)),
    # state kinds sharded over the data-parallel replicas
    (SMALL, SMALL_MIX, Parallel(2, 1, 2, shard_kinds=2), Parallel(2, 1, 4, shard_kinds=2)),
    (SMALL, SMALL_MIX, Parallel(4, 2, 2, shard_kinds=2), Parallel(2, 2, 1)),
    (SMALL, SMALL_MIX, Parallel(2, 1, 1), Parallel(3, 2, 3, shard_kinds=3)),
    (SMALL, SMALL_MIX, Parallel(2, 1, 3, shard_kinds=1, qkv_layout=1), Parallel(1, 2, 5, shard_kinds=2, w_transposed=1)),
    (ODD, ODD_MIX, Parallel(3, 1, 2, shard_kinds=2), Parallel(4, 1, 3, shard_kinds=3)),
    (WIDE, H.synth.MIX_GPT, Parallel(2, 2, 2, shard_kinds=14), Parallel(4, 1, 4, shard_kinds=14)),
    # arbitrary layer -> stage maps (interleaved pipeline chunks; a stage without layers)
    (SMALL, SMALL_MIX, Parallel(2, 2, 1, layer_stage=(0, 1, 0, 1)), Parallel(3, 2, 1)),
    (SMALL, SMALL_MIX, Parallel(4, 1, 1), Parallel(2, 3, 2, layer_stage=(2, 0, 0, 2), shard_kinds=2)),
    (SMALL, SMALL_MIX, Parallel(2, 2, 1, layer_stage=(1, 0, 1, 0)), Parallel(2, 4, 1, layer_stage=(3, 2, 1, 0))),
]


@pytest.mark.parametrize("model,mix,src,dst", PAIRS)
@pytest.mark.parametrize("how", ["boxes", "tiles"])
def test_plan_interpreted_on_cpu_matches_oracle(model, mix, src, dst, how):
    """The copy list (and its tiling) moves exactly the bytes the oracle's definition moves, writes every
    destination tensor byte exactly once and touches nothing else."""
    src_bufs = H.np_bufs(H.make_src_bufs(model, src, 17, mix))
    want = oreshard.reshard(model, src, dst, src_bufs)
    plan = plan_for(model, src, dst, opts=dict(tile_bytes=4096) if how == "tiles" else None)
    got = [np.full(plan.buffer_bytes(1, r), H.POISON, dtype=np.uint8) for r in range(dst.n_ranks)]
    cover = [np.zeros(len(g), dtype=np.int32) for g in got]
    (host_exec.run_boxes if how == "boxes" else host_exec.run_tiles)(plan, src_bufs, got, cover)
    for r in range(dst.n_ranks):
        assert np.array_equal(got[r], want[r]), r
        expect_cover = np.zeros(len(got[r]), dtype=np.int32)
        for e in spec.rank_manifest(model, dst, r)[0]:
            d = H.desc_of(e)
            expect_cover[d.offset:d.offset + d.nbytes] = 1
        assert np.array_equal(cover[r], expect_cover), r
    s = plan.stats()
    assert s["bytes_written"] == oreshard.state_bytes(model, dst)
    if dst.D == 1 or dst.shard_kinds == (1 << len(model.state_elem_bytes)) - 1:
        assert s["bytes_read"] == s["bytes_written"] - s["bytes_fill"]
    else:       # replicas fed by one multicast move read their source once
        assert s["bytes_read"] <= s["bytes_written"] - s["bytes_fill"]


# ---- closed forms of the plan -------------------------------------------------------------------
@pytest.mark.parametrize("T,Tn", [(2, 3), (2, 4), (4, 2), (3, 4), (8, 1), (1, 8), (6, 4), (4, 4), (12, 8)])
def test_pieces_per_sliced_tensor(T, Tn):
    """Re-slicing one axis from T to T' equal parts cuts it at the union of both sets of cut points:
    T + T' - gcd(T, T') pieces (figure 6: 2 -> 3 gives 4, each old half cut in two)."""
    model = Model(n_layers=1, hidden=48, n_heads=24, ffn=96, vocab_true=48, max_pos=2, state_elem_bytes=(4,))
    plan = plan_for(model, Parallel(T, 1, 1), Parallel(Tn, 1, 1))
    per = T + Tn - math.gcd(T, Tn)
    n_sliced, n_repl = 7, 9               # 7 sliced tensors; 9 replicated ones (pos emb, 4+2 LN, 2 biases)
    assert plan.stats()["n_pieces"] == n_sliced * per + n_repl * Tn
    if (T, Tn) == (2, 3):
        tid = spec.tensor_id(spec.FC1_B, 0)
        bx = [b for b in plan.boxes() if b.tensor_id == tid]
        assert sorted((b.src_rank, b.dst_rank, b.run_bytes) for b in bx) == \
            [(0, 0, 128), (0, 1, 64), (1, 1, 64), (1, 2, 128)]


def test_unchanged_configuration_is_one_copy_per_rank():
    """Redeployment with the same configuration (paper section 6.3): each rank buffer moves whole."""
    model, par = H.GPT_1_3B, Parallel(4, 2, 1)
    plan = plan_for(model, par, par)
    boxes = plan.boxes()
    assert len(boxes) == par.n_ranks
    for r, b in enumerate(boxes):
        assert (b.src_rank, b.dst_rank, b.ndim, b.src_off, b.dst_off) == (r, r, 0, 0, 0)
        assert b.run_bytes == plan.buffer_bytes(0, r)
    assert plan.stats()["bytes_cross_rank"] == 0


def test_pipeline_only_change_moves_whole_sub_tensors():
    """A change of P alone re-partitions without splitting or merging (paper section 6.7)."""
    model = H.GPT_1_3B
    src, dst = Parallel(4, 2, 1), Parallel(4, 4, 1)
    plan = plan_for(model, src, dst)
    n_entries = sum(len(spec.rank_manifest(model, dst, r)[0]) for r in range(dst.n_ranks))
    assert plan.stats()["n_pieces"] == n_entries
    assert all(b.ndim == 0 and b.kind == B.BOX_COPY for b in plan.boxes())
    # neighbours merge: per destination rank one run per state kind
    assert plan.stats()["n_boxes"] == dst.n_ranks * len(model.state_elem_bytes)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_byte_totals_of_the_five_workloads(cfg):
    model, src, dst, _, _ = H.CONFIGS[cfg]
    s = plan_for(model, src, dst).stats()
    assert s["bytes_written"] == oreshard.state_bytes(model, dst)
    assert s["bytes_read"] == s["bytes_written"] - s["bytes_fill"]
    if cfg == 3:    # replicas are read once: nothing is read twice although the source holds two copies
        assert s["bytes_read"] == oreshard.state_bytes(model, dst) < oreshard.state_bytes(model, src)
    if cfg == 4:
        assert s["bytes_written"] == 93_161_635_840      # 6,654,402,560 parameters x 14 B, nothing replicated at T'=1
    if cfg == 5:    # 384 new padding rows of 3072 elements, 14 bytes each
        assert s["bytes_fill"] == 384 * 3072 * 14
    else:
        assert s["bytes_fill"] == 0


def test_scale_out_writes_every_replica():
    """More data-parallel replicas: bytes written grow with D' (paper section 6.7)."""
    model = H.GPT_1_3B
    one = plan_for(model, Parallel(4, 2, 1), Parallel(4, 2, 1)).stats()
    two = plan_for(model, Parallel(4, 2, 1), Parallel(4, 2, 2)).stats()
    assert two["bytes_written"] == 2 * one["bytes_written"]
    # ... but both replicas are written from one read of the source (multicast moves)
    assert two["bytes_read"] == one["bytes_read"]
    plan = plan_for(model, Parallel(4, 2, 1), Parallel(4, 2, 2))
    assert all(b.n_dst == 2 and b.dst_rank_stride == 4 for b in plan.boxes())
    # replicas that prefer different (local) sources are planned separately: nothing crosses buffers
    s = plan_for(model, Parallel(2, 1, 2), Parallel(2, 1, 2)).stats()
    assert s["bytes_cross_rank"] == 0 and s["bytes_read"] == s["bytes_written"]


@pytest.mark.parametrize("src,dst", [(Parallel(1, 1, 4), Parallel(1, 1, 8)), (Parallel(2, 1, 2), Parallel(2, 1, 12)),
                                     (Parallel(2, 2, 2), Parallel(4, 1, 3)), (Parallel(2, 1, 3), Parallel(2, 1, 2))])
def test_share_reads_reads_every_piece_once(src, dst):
    """Option share_reads: a replica group reads what its first member reads - same bytes land, each
    distinct piece is read once per multicast move (at most max_multicast destinations each)."""
    model, mix = SMALL, SMALL_MIX
    src_bufs = H.np_bufs(H.make_src_bufs(model, src, 23, mix))
    want = oreshard.reshard(model, src, dst, src_bufs)
    local = plan_for(model, src, dst).stats()
    plan = plan_for(model, src, dst, opts=dict(share_reads=1))
    for how in (host_exec.run_boxes, host_exec.run_tiles):
        got = [np.full(plan.buffer_bytes(1, r), H.POISON, dtype=np.uint8) for r in range(dst.n_ranks)]
        how(plan, src_bufs, got)
        assert all(np.array_equal(g, w) for g, w in zip(got, want))
    s = plan.stats()
    one_replica = oreshard.state_bytes(model, Parallel(dst.T, dst.P, 1))
    assert s["bytes_written"] == local["bytes_written"] == dst.D * one_replica
    assert s["bytes_read"] == -(-dst.D // 8) * one_replica <= local["bytes_read"]
    assert s["bytes_cross_rank"] >= local["bytes_cross_rank"]      # the price: locality is given up
    assert {b.n_dst for b in plan.boxes()} == ({8, dst.D % 8} - {0} if dst.D > 8 else {dst.D})


@pytest.mark.parametrize("model,mix,src,dst", PAIRS)
def test_traffic_matrix_accounts_for_every_moved_byte(model, mix, src, dst):
    """tpx_traffic: column sums = bytes each destination rank receives (its tensor bytes minus zero fill), the
    off-diagonal sum = bytes_cross_rank, and lost or absent pairs are zero."""
    plan = plan_for(model, src, dst)
    m = plan.traffic()
    s = plan.stats()
    assert len(m) == src.n_ranks and all(len(row) == dst.n_ranks for row in m)
    assert sum(map(sum, m)) == s["bytes_written"] - s["bytes_fill"]
    assert sum(m[i][j] for i in range(src.n_ranks) for j in range(dst.n_ranks) if i != j) == s["bytes_cross_rank"]
    want = [np.zeros(dst.n_ranks, dtype=np.int64) for _ in range(src.n_ranks)]
    for b in plan.boxes():
        if b.kind != B.BOX_FILL:
            n = b.run_bytes * int(np.prod([b.extent[k] for k in range(b.ndim)], dtype=np.int64))
            for k in range(b.n_dst):
                want[b.src_rank][b.dst_rank + k * b.dst_rank_stride] += n
    assert [list(map(int, row)) for row in want] == m
    if model.vocab_divisor == 0:          # no zero fill: every destination receives exactly its tensor bytes
        for j in range(dst.n_ranks):
            mine = sum(H.desc_of(e).nbytes for e in spec.rank_manifest(model, dst, j)[0])
            assert sum(m[i][j] for i in range(src.n_ranks)) == mine


def test_traffic_of_a_pipeline_only_change_is_block_structured():
    """(4,2,1) -> (4,4,1): destination stage p' of tensor-parallel rank t receives only from old stage p'//2, same t."""
    plan = plan_for(H.GPT_1_3B, Parallel(4, 2, 1), Parallel(4, 4, 1))
    m = plan.traffic()
    for i in range(8):
        for j in range(16):
            assert (m[i][j] > 0) == (i % 4 == j % 4 and i // 4 == (j // 4) // 2), (i, j)


def _identity_maps(model, par, mix):
    """Per rank: int64 array with a unique id (tensor, kind, position) per element slot of 2 bytes."""
    out = []
    for r in range(par.n_ranks):
        entries, n = spec.rank_manifest(model, par, r)
        ident = np.full(n // 2, -1, dtype=np.int64)
        for e in entries:
            d = H.desc_of(e)
            lin = H.synth.linear_index(d, "cpu").reshape(-1).numpy()
            key = (e.tensor_id * 8 + e.kind) * (1 << 40) + lin
            per = e.elem_bytes // 2
            ident[d.offset // 2:d.offset // 2 + lin.size * per] = np.repeat(key, per)
        out.append(ident)
    return out


@pytest.mark.parametrize("src,dst", [(Parallel(2, 1, 2), Parallel(4, 1, 1)), (Parallel(4, 2, 2), Parallel(2, 2, 1)),
                                     (Parallel(2, 2, 1), Parallel(2, 1, 2)), (Parallel(3, 1, 1), Parallel(2, 2, 1)),
                                     (Parallel(4, 4, 2), Parallel(2, 4, 1, stage_first_layer=(0, 1, 1, 3, 4)))])
def test_cross_rank_bytes_equal_brute_force_minimum(src, dst):
    """Element by element: a destination element must cross buffers only if no source buffer with the
    destination's own index holds it. The plan's cross-rank byte count equals that minimum."""
    model = Model(n_layers=4, hidden=24, n_heads=12, ffn=48, vocab_true=36, max_pos=5, state_elem_bytes=(4, 2))
    s_id, d_id = _identity_maps(model, src, None), _identity_maps(model, dst, None)
    must_cross = 0
    for r in range(dst.n_ranks):
        keys = d_id[r][d_id[r] >= 0]
        local = s_id[r] if r < src.n_ranks else np.zeros(0, dtype=np.int64)
        must_cross += 2 * int(np.count_nonzero(~np.isin(keys, local)))
    assert plan_for(model, src, dst).stats()["bytes_cross_rank"] == must_cross


# ---- failure recovery (paper section 5.3) -------------------------------------------------------
def test_lost_ranks_are_avoided_when_a_replica_survives():
    model, mix = SMALL, SMALL_MIX
    src, dst = Parallel(2, 2, 2), Parallel(2, 1, 1)
    alive = [1] * src.n_ranks
    for t in range(2):                       # lose replica d=0 of stage 0 and replica d=1 of stage 1
        alive[spec.rank_of(src, t, 0, 0)] = 0
        alive[spec.rank_of(src, t, 1, 1)] = 0
    plan = plan_for(model, src, dst, rank_alive=alive)
    assert all(alive[b.src_rank] for b in plan.boxes())
    src_bufs = H.np_bufs(H.make_src_bufs(model, src, 5, mix))
    want = oreshard.reshard(model, src, dst, src_bufs)
    for r, a in enumerate(alive):
        if not a:
            src_bufs[r][:] = 0xEE           # lost buffers hold garbage
    got = [np.full(plan.buffer_bytes(1, r), H.POISON, dtype=np.uint8) for r in range(dst.n_ranks)]
    host_exec.run_boxes(plan, src_bufs, got)
    assert all(np.array_equal(g, w) for g, w in zip(got, want))


def test_unrecoverable_when_no_holder_survives():
    src = Parallel(2, 2, 2)
    alive = [1] * src.n_ranks
    alive[spec.rank_of(src, 1, 1, 0)] = alive[spec.rank_of(src, 1, 1, 1)] = 0
    with pytest.raises(tpx.TpxError) as ei:
        plan_for(SMALL, src, Parallel(1, 1, 1), rank_alive=alive)
    assert ei.value.status == B.TPX_ERR_UNRECOVERABLE


@pytest.mark.parametrize("lost", [4, 8, 12])
def test_rebuild_only_the_lost_ranks_of_sixteen(lost):
    """Section 5.3 / 6.4 shape: (T,P,D) = (4,2,2), 16 ranks, some lost.  Only the lost ranks are rebuilt (the
    destination mask), from the surviving replica of each; with both replicas of a (t, p) share gone the state
    is unrecoverable."""
    model, mix = SMALL, SMALL_MIX
    cfg = Parallel(4, 2, 2)
    rng = np.random.default_rng(lost)
    # lose `lost` ranks but never both replicas of one (t, p) share
    shares = [(t, p) for p in range(2) for t in range(4)]
    gone = set()
    if lost <= 8:
        for t, p in [shares[i] for i in rng.permutation(8)[:lost]]:
            gone.add(spec.rank_of(cfg, t, p, int(rng.integers(2))))
    else:
        for t, p in shares:
            gone.add(spec.rank_of(cfg, t, p, int(rng.integers(2))))
        gone |= set(int(x) for x in rng.permutation([r for r in range(16) if r not in gone])[:lost - 8])
    alive = [0 if r in gone else 1 for r in range(16)]
    need = [1 - a for a in alive]
    if lost > 8:
        with pytest.raises(tpx.TpxError) as ei:
            plan_for(model, cfg, cfg, dst_alive=need, rank_alive=alive)
        assert ei.value.status == B.TPX_ERR_UNRECOVERABLE
        return
    plan = plan_for(model, cfg, cfg, dst_alive=need, rank_alive=alive)
    boxes = plan.boxes()
    assert all(alive[b.src_rank] and need[b.dst_rank] for b in boxes)
    src_bufs = H.np_bufs(H.make_src_bufs(model, cfg, 5, mix))
    want = oreshard.reshard(model, cfg, cfg, src_bufs)
    for r in gone:
        src_bufs[r][:] = 0xEE
    got = [np.full(plan.buffer_bytes(1, r), H.POISON, dtype=np.uint8) for r in range(16)]
    host_exec.run_tiles(plan, src_bufs, got)
    for r in range(16):
        if need[r]:
            assert np.array_equal(got[r], want[r]), r
        else:
            assert (got[r] == H.POISON).all(), r                      # survivors are left alone
    s = plan.stats()
    rank_bytes = [sum(H.desc_of(e).nbytes for e in spec.rank_manifest(model, cfg, r)[0]) for r in range(16)]
    rebuilt = sum(rank_bytes[r] for r in gone)
    assert s["bytes_written"] == rebuilt == s["bytes_read"] == s["bytes_cross_rank"]
    m = plan.traffic()
    assert all(sum(m[i][j] for i in range(16)) == (rank_bytes[j] if need[j] else 0) for j in range(16))


def test_sharded_kinds_have_no_replica_to_recover_from():
    """A state kind cut over the replicas is stored once: losing one rank loses its chunk, while the kinds
    that are still replicated survive the same loss."""
    src = Parallel(2, 1, 2, shard_kinds=2)
    alive = [1] * src.n_ranks
    alive[spec.rank_of(src, 0, 0, 1)] = 0
    with pytest.raises(tpx.TpxError) as ei:
        plan_for(SMALL, src, Parallel(1, 1, 1), rank_alive=alive)
    assert ei.value.status == B.TPX_ERR_UNRECOVERABLE
    plan = plan_for(SMALL, Parallel(2, 1, 2), Parallel(1, 1, 1), rank_alive=alive)      # fully replicated: fine
    assert all(alive[b.src_rank] for b in plan.boxes())
    with pytest.raises(tpx.TpxError) as ei:                                              # a kind the model lacks
        plan_for(SMALL, Parallel(2, 1, 2, shard_kinds=4), Parallel(1, 1, 1))
    assert ei.value.status == B.TPX_ERR_INVALID_ARG
    with pytest.raises(tpx.TpxError) as ei:                                              # a layer on a stage that does not exist
        tpx.tpx_plan(mk(SMALL), dict(T=2, P=2, D=1, layer_stage=(0, 1, 2, 0)), pk(Parallel(1, 1, 1)))
    assert ei.value.status == B.TPX_ERR_BAD_STAGE_MAP


# ---- error codes ----------------------------------------------------------------------------------
def test_error_codes():
    m = mk(SMALL)
    def st(fn):
        with pytest.raises(tpx.TpxError) as ei:
            fn()
        return ei.value.status
    assert st(lambda: tpx.tpx_plan(m, dict(T=5, P=1, D=1), dict(T=1, P=1, D=1))) == B.TPX_ERR_INDIVISIBLE
    assert st(lambda: tpx.tpx_plan(m, dict(T=1, P=3, D=1), dict(T=1, P=1, D=1))) == B.TPX_ERR_INDIVISIBLE
    assert st(lambda: tpx.tpx_plan(m, dict(T=1, P=2, D=1, stage_first_layer=(0, 3, 2)), dict(T=1, P=1, D=1))) == B.TPX_ERR_BAD_STAGE_MAP
    assert st(lambda: tpx.tpx_plan(m, dict(T=1, P=2, D=1, stage_first_layer=(1, 2, 4)), dict(T=1, P=1, D=1))) == B.TPX_ERR_BAD_STAGE_MAP
    assert st(lambda: tpx.tpx_plan(m, dict(T=0, P=1, D=1), dict(T=1, P=1, D=1))) == B.TPX_ERR_INVALID_ARG
    assert st(lambda: tpx.tpx_plan(m, dict(T=2, P=4, D=32), dict(T=1, P=1, D=1))) == B.TPX_ERR_INVALID_ARG
    bad = dict(m, state_elem_bytes=(3,))
    assert st(lambda: tpx.tpx_plan(bad, dict(T=1, P=1, D=1), dict(T=1, P=1, D=1))) == B.TPX_ERR_INVALID_ARG
    odd_vocab = dict(m, vocab_true=37)
    assert st(lambda: tpx.tpx_plan(odd_vocab, dict(T=2, P=1, D=1), dict(T=1, P=1, D=1))) == B.TPX_ERR_INDIVISIBLE
    assert st(lambda: tpx.tpx_set_option("no_such_option", 1)) == B.TPX_ERR_INVALID_ARG
    assert st(lambda: tpx.tpx_set_option("tile_bytes", 4096)) == B.TPX_ERR_INVALID_ARG      # a plan option, not a knob
    assert st(lambda: tpx.tpx_set_option("streams", 0)) == B.TPX_ERR_INVALID_ARG
    assert st(lambda: tpx.tpx_set_option("chunk", 5000)) == B.TPX_ERR_INVALID_ARG
    assert st(lambda: tpx.tpx_set_option("occupancy", 17)) == B.TPX_ERR_INVALID_ARG
    one = dict(T=1, P=1, D=1)
    for bad_opts in (dict(tile_bytes=5000), dict(tile_bytes=2048), dict(max_multicast=129), dict(share_reads=2), dict(tiles=1),
                     dict(pack_bytes=65537), dict(tile_bytes=4096, pack_bytes=8192)):
        assert st(lambda: tpx.tpx_plan(m, one, one, bad_opts)) == B.TPX_ERR_INVALID_ARG
    # lists whose length the library cannot check are checked by the binding
    assert st(lambda: tpx.tpx_plan(m, dict(T=1, P=2, D=1, stage_first_layer=(0, 2)), one)) == B.TPX_ERR_INVALID_ARG
    assert st(lambda: tpx.tpx_plan(m, dict(T=2, P=1, D=2, rank_alive=[1, 1, 1]), one)) == B.TPX_ERR_INVALID_ARG
    assert st(lambda: tpx.tpx_plan(m, dict(T=1, P=2, D=1, layer_stage=(0, 1, 1)), one)) == B.TPX_ERR_INVALID_ARG
    assert st(lambda: tpx.tpx_plan_ptc([[]], [[]], src_bytes=[0, 0])) == B.TPX_ERR_INVALID_ARG
    assert st(lambda: tpx.tpx_plan_ptc([[]], [[]], src_alive=[1, 1])) == B.TPX_ERR_INVALID_ARG
    assert B._lib.tpx_plan(None, None, None, None, None) == B.TPX_ERR_INVALID_ARG
    assert B._lib.tpx_execute(None, None, None, None, None) == B.TPX_ERR_INVALID_ARG
    assert b"NULL" in B._lib.tpx_last_error()
    assert B._lib.tpx_num_buffers(None, 0) == 0 and B._lib.tpx_workspace_bytes(None) == 0
    B._lib.tpx_free(None)


def test_tiles_are_bounded_and_vector_aligned_on_the_headline_workload():
    model, src, dst, _, _ = H.CONFIGS[4]
    plan = plan_for(model, src, dst)
    s = plan.stats()
    assert s["n_tiles"] == plan.num_tiles() and plan.workspace_bytes() < (1 << 20)     # tiles are derived, not stored
    total = 0
    for i in range(0, plan.num_tiles(), 997):
        t = B.tpx_tile()
        B._check(B._lib.tpx_get_tile(plan._h, i, t))
        assert t.unit_log2 == 4 and t.kind in (B.TILE_COPY, B.TILE_MERGE, B.TILE_PACK)
        assert t.nrows * t.run_units * 16 <= 131072
        total += 1
    assert total > 300


def pack_tiles(plan):
    """The PACK tiles of a plan: they are its last tiles."""
    out = []
    for i in range(plan.num_tiles() - 1, -1, -1):
        t = B.tpx_tile()
        B._check(B._lib.tpx_get_tile(plan._h, i, t))
        if t.kind != B.TILE_PACK:
            break
        out.append(t)
    return out[::-1]


def test_short_moves_share_pack_tiles():
    """BERT-large shape, T 4 -> 8: biases and LayerNorm vectors (a few KiB each) are a few percent of the tiles when every one
    has its own; packed, up to 64 of them that go to the same destination buffer share a tile.  Everything else about the plan
    stays as it is, and the packed plan interpreted on the CPU still writes every destination byte exactly once."""
    import bench
    mk_, s_, d_, _, _ = bench.WORKLOADS["bert-large_(4,1,1)->(8,1,1)"]
    apart = tpx.tpx_plan(mk_, s_, d_, dict(pack_bytes=1))
    packed = tpx.tpx_plan(mk_, s_, d_)
    a, p = apart.stats(), packed.stats()
    assert not pack_tiles(apart) and len(apart.segments()) == 0
    assert {k: a[k] for k in a if k not in ("n_tiles", "plan_ns")} == {k: p[k] for k in p if k not in ("n_tiles", "plan_ns")}
    packs = pack_tiles(packed)
    segs = packed.segments()
    moved = sum(t.n_seg for t in packs)
    assert a["n_tiles"] - p["n_tiles"] == moved - len(packs) and moved > 2000 and len(packs) <= moved // 8
    assert {t.dst_rank for t in packs} == set(range(8)) and all(t.run_units * 16 <= 65536 and t.n_seg <= 64 for t in packs)
    assert all(segs[t.seg_first + g].units * 16 <= 16384 for t in packs for g in range(t.n_seg))
    # a small model through the CPU interpreter: packed and unpacked plans write the same bytes, each exactly once
    for opts in (None, dict(pack_bytes=1), dict(pack_bytes=512), dict(tile_bytes=4096, pack_bytes=4096)):
        src, dst = Parallel(4, 1, 1), Parallel(2, 2, 3)
        plan = plan_for(WIDE, src, dst, opts=opts)
        assert bool(pack_tiles(plan)) == (opts != dict(pack_bytes=1))
        src_bufs = H.np_bufs(H.make_src_bufs(WIDE, src, 7, H.synth.MIX_GPT))
        want = oreshard.reshard(WIDE, src, dst, src_bufs)
        got = [np.full(plan.buffer_bytes(1, r), H.POISON, dtype=np.uint8) for r in range(plan.num_buffers(1))]
        cover = [np.zeros(len(g), dtype=np.int32) for g in got]
        host_exec.run_tiles(plan, src_bufs, got, cover)
        assert all(np.array_equal(g, w) for g, w in zip(got, want))
        assert all(c.max() <= 1 for c in cover)


def test_row_parallel_merges_become_merge_tiles():
    """T 8 -> 1: every row-parallel weight (attention projection, MLP down-projection) is merged from 8 column
    blocks; its tiles write whole destination rows and read 8 segments (merge of algorithm 1, inside the tile)."""
    model, src, dst, _, _ = H.CONFIGS[4]
    plan = plan_for(model, src, dst)
    segs = plan.segments()
    n_packed = sum(t.n_seg for t in pack_tiles(plan))
    assert len(segs) - n_packed == model.n_layers * len(model.state_elem_bytes) * 2 * 8      # the segments of the merges come first
    assert sorted({g.src_rank for g in segs[:len(segs) - n_packed]}) == list(range(8))
    merge_bytes = 0
    for i in range(0, plan.num_tiles(), 101):
        t = B.tpx_tile()
        B._check(B._lib.tpx_get_tile(plan._h, i, t))
        if t.kind == B.TILE_MERGE:
            assert t.n_seg == 8 and t.n_seg * t.seg_units == t.run_units and t.dst_pitch == t.run_units * 16
            merge_bytes += 1
    assert merge_bytes > 500
    # a 3 -> 4 re-slicing has unequal pieces per destination row (thirds against quarters, in twelfths: new quarter 1 = 1 + 2,
    # quarter 2 = 2 + 1): those merges carry each segment's own width; quarters 0 and 3 lie inside one third (plain copies)
    model5, src5, dst5, _, _ = H.CONFIGS[5]
    plan5 = plan_for(model5, src5, dst5)
    segs5 = plan5.segments()
    n_packed5 = sum(t.n_seg for t in pack_tiles(plan5))
    assert len(segs5) - n_packed5 == model5.n_layers * len(model5.state_elem_bytes) * 2 * 2 * 2     # 2 weights x 2 middle quarters x 2 pieces
    irregular = 0
    for i in range(0, plan5.num_tiles(), 53):
        t = B.tpx_tile()
        B._check(B._lib.tpx_get_tile(plan5._h, i, t))
        if t.kind == B.TILE_MERGE:
            w = [segs5[t.seg_first + g].units for g in range(t.n_seg)]
            assert t.seg_units == 0 and t.n_seg == 2 and sum(w) == t.run_units and sorted(w) == [t.run_units // 3, 2 * t.run_units // 3]
            irregular += 1
    assert irregular > 100


def test_command_line_front_end():
    import json
    import subprocess
    import sys
    base = [sys.executable, "-m", "paper_2312_05181_amd"]
    args = ["--layers", "2", "--hidden", "256", "--heads", "4", "--ffn", "1024", "--vocab", "1024", "--state-bytes", "4,4,4",
            "--src", "2,1,1", "--dst", "4,2,1"]
    out = subprocess.run(base + ["plan"] + args, cwd=ROOT, capture_output=True, text=True, check=True).stdout
    st = json.loads(out)
    assert st["bytes_written"] == oreshard.state_bytes(H.TINY, Parallel(4, 2, 1)) and len(st["dst_buffer_bytes"]) == 8
    out = subprocess.run(base + ["manifest"] + args + ["--side", "dst", "--rank", "7"], cwd=ROOT, capture_output=True, text=True, check=True).stdout
    assert "/7/layer1/attention.query_key_value.weight[kind 0]" in out and "final_layernorm.bias" in out
    bad = subprocess.run(base + ["plan"] + args[:-1] + ["3,1,1"], cwd=ROOT, capture_output=True, text=True)
    assert bad.returncode == 1 and "tpx status -2" in bad.stderr


def test_package_imports_without_the_library_and_fails_loudly_on_use(tmp_path):
    """A tree without libtpx.so: the package (and so its build module) still imports; any use raises."""
    import shutil
    import subprocess
    import sys
    pkg = tmp_path / "paper_2312_05181_amd"
    pkg.mkdir()
    for f in ("__init__.py", "binding.py", "build.py"):
        shutil.copy(os.path.join(ROOT, "paper_2312_05181_amd", f), pkg / f)
    code = ("import paper_2312_05181_amd as t, paper_2312_05181_amd.build\n"
            "try:\n    t.tpx_plan\nexcept ImportError as e:\n    print('LOUD', e)\n")
    out = subprocess.run([sys.executable, "-c", code], cwd=tmp_path, capture_output=True, text=True, check=True).stdout
    assert "LOUD" in out and "no CPU fallback" in out
