"""Collections given explicitly (paper section 4.3: the same three functions express expert parallelism,
sequence parallelism and other strategies): the generic oracle against the value function, and libtpx's
planner (interpreted on the CPU) against the generic oracle."""
import numpy as np
import pytest
import torch

import paper_2312_05181_amd as tpx
import paper_2312_05181_amd.binding as B
import synth
from oracle import reshard as oreshard
from oracle import spec
from tests import helpers as H
from tests import host_exec

MIX = ((2, "bf16w"), (4, "n02"), (4, "m"), (4, "v"))


def pack(boxes):
    """boxes: per rank a list of (tensor_id, kind, elem_bytes, full_shape, lo, hi, perm); assigns 256-aligned
    offsets in list order.  Returns per rank (entries, nbytes)."""
    out = []
    for per_rank in boxes:
        off, entries = 0, []
        for tid, kind, eb, full, lo, hi, perm in per_rank:
            off = -(-off // 256) * 256
            entries.append(spec.Entry(tid, kind, eb, off, tuple(full), tuple(lo), tuple(hi), tuple(perm), 0, -1))
            off += int(np.prod([h - l for l, h in zip(lo, hi)])) * eb
        out.append((entries, -(-off // 256) * 256))
    return out


def even(n, parts, i):
    return (n * i) // parts, (n * (i + 1)) // parts


# ---- the collections ---------------------------------------------------------------------------------
def experts(n_ranks, tp=1, n_experts=8, h=32, f=64):
    """Expert parallelism: phi groups whole expert tensors (sigma is the identity); optionally each expert's
    matrices are also tensor-parallel (tp) on the ffn axis.  Rank = ep_rank * tp + t."""
    ranks = []
    ep = n_ranks // tp
    for r in range(n_ranks):
        e_lo, e_hi = even(n_experts, ep, r // tp)
        t = r % tp
        per = []
        for kind, eb in enumerate((2, 4, 4, 4)):
            for e in range(e_lo, e_hi):
                a, b = even(f, tp, t)
                per.append((2 * e, kind, eb, (f, h), (a, 0), (b, h), (0, 1)))          # up-projection, rows cut
                per.append((2 * e + 1, kind, eb, (h, f), (0, a), (h, b), (0, 1)))      # down-projection, columns cut
        ranks.append(per)
    return pack(ranks)


def sequence(n_ranks, batch=4, seq=64, hidden=48):
    """Sequence parallelism: sigma slices a sample tensor [batch, seq, hidden] along seq."""
    ranks = []
    for r in range(n_ranks):
        a, b = even(seq, n_ranks, r)
        ranks.append([(0, 0, 2, (batch, seq, hidden), (0, a, 0), (batch, b, hidden), (0, 1, 2))])
    return pack(ranks)


def sharded_optimizer(n_ranks, n=100_003):
    """Optimizer state flattened and cut into contiguous chunks, one per data-parallel rank (uneven sizes)."""
    ranks = []
    for r in range(n_ranks):
        a, b = even(n, n_ranks, r)
        ranks.append([(0, k, 4, (n,), (a,), (b,), (0,)) for k in (1, 2, 3)])
    return pack(ranks)


def grid2d(rows, cols, shape=(64, 96)):
    """Two-dimensional tensor parallelism: a rows x cols grid of blocks; rank = i * cols + j."""
    ranks = []
    for i in range(rows):
        for j in range(cols):
            a, b = even(shape[0], rows, i)
            c, d = even(shape[1], cols, j)
            ranks.append([(0, k, eb, shape, (a, c), (b, d), (0, 1)) for k, eb in enumerate((2, 4))])
    return pack(ranks)


def replicated(n_copies, base):
    return [base[i % len(base)] for i in range(n_copies * len(base))]


CASES = {
    "experts 2 -> 4 ranks": (experts(2), experts(4)),
    "experts 4 -> 2 ranks": (experts(4), experts(2)),
    "experts ep2 -> ep2 x tp2": (experts(2), experts(4, tp=2)),
    "experts ep4 x tp2 -> ep2": (experts(8, tp=2), experts(2)),
    "sequence 2 -> 4": (sequence(2), sequence(4)),
    "sequence 4 -> 1": (sequence(4), sequence(1)),
    "sequence 3 -> 2 (uneven pieces)": (sequence(3, seq=66), sequence(2, seq=66)),
    "sharded optimizer 3 -> 4": (sharded_optimizer(3), sharded_optimizer(4)),
    "sharded optimizer 4 -> 1": (sharded_optimizer(4), sharded_optimizer(1)),
    "2-D grid 2x2 -> 1x4": (grid2d(2, 2), grid2d(1, 4)),
    "2-D grid 2x2 -> 4x1": (grid2d(2, 2), grid2d(4, 1)),
    "2-D grid 1x4 -> 2x3": (grid2d(1, 4), grid2d(2, 3)),
    "experts 2 -> 2 replicas of 2": (experts(2), replicated(2, experts(2))),
}


def src_buffers(man, seed, device="cpu"):
    bufs = []
    for entries, n in man:
        b = torch.full((n,), H.SRC_GAP, dtype=torch.uint8, device=device)
        synth.fill_buffer(b, [H.desc_of(e) for e in entries], seed, MIX)
        bufs.append(b)
    return bufs


def closed_form(man, seed, device="cpu"):
    bufs = []
    for entries, n in man:
        b = torch.full((n,), H.POISON, dtype=torch.uint8, device=device)
        synth.fill_buffer(b, [H.desc_of(e) for e in entries], seed, MIX)
        bufs.append(b)
    return bufs


def plan_of(src, dst, **kw):
    return tpx.tpx_plan_ptc([[H.desc_of(e) for e in ent] for ent, _ in src], [[H.desc_of(e) for e in ent] for ent, _ in dst],
                            src_bytes=[n for _, n in src], dst_bytes=[n for _, n in dst], **kw)


@pytest.mark.parametrize("name", list(CASES))
def test_generic_oracle_matches_value_function_and_round_trips(name):
    src, dst = CASES[name]
    a = H.np_bufs(src_buffers(src, 5))
    out = oreshard.reshard_ptc(src, dst, a)
    want = H.np_bufs(closed_form(dst, 5))
    assert all(np.array_equal(x, y) for x, y in zip(out, want))
    back = oreshard.reshard_ptc(dst, src, out)
    for r, (entries, _) in enumerate(src):
        for e in entries:
            d = H.desc_of(e)
            assert np.array_equal(back[r][d.offset:d.offset + d.nbytes], a[r][d.offset:d.offset + d.nbytes])


@pytest.mark.parametrize("how", ["boxes", "tiles"])
@pytest.mark.parametrize("name", list(CASES))
def test_generic_plan_matches_oracle(name, how):
    src, dst = CASES[name]
    a = H.np_bufs(src_buffers(src, 7))
    want = oreshard.reshard_ptc(src, dst, a)
    plan = plan_of(src, dst, opts=dict(tile_bytes=4096))
    got = [np.full(n, H.POISON, dtype=np.uint8) for _, n in dst]
    cover = [np.zeros(n, dtype=np.int32) for _, n in dst]
    (host_exec.run_boxes if how == "boxes" else host_exec.run_tiles)(plan, a, got, cover)
    for r, (entries, n) in enumerate(dst):
        assert plan.buffer_bytes(1, r) == n
        assert np.array_equal(got[r], want[r]), r
        expect = np.zeros(n, dtype=np.int32)
        for e in entries:
            d = H.desc_of(e)
            expect[d.offset:d.offset + d.nbytes] = 1
        assert np.array_equal(cover[r], expect)


def test_expert_regrouping_moves_whole_tensors():
    """Expert parallelism changes only phi: no sub-tensor is split, and neighbours merge into long runs."""
    plan = plan_of(*CASES["experts 2 -> 4 ranks"])
    assert all(b.kind == B.BOX_COPY and b.ndim == 0 for b in plan.boxes())
    assert plan.stats()["n_boxes"] == 4 * 4          # one run per destination rank and state kind


def test_identical_destination_ranks_are_replicas():
    plan = plan_of(*CASES["experts 2 -> 2 replicas of 2"])
    s = plan.stats()
    assert s["bytes_written"] == 2 * s["bytes_read"]
    assert all(b.n_dst == 2 and b.dst_rank_stride == 2 for b in plan.boxes())


def test_generic_errors():
    def st(fn):
        with pytest.raises(tpx.TpxError) as ei:
            fn()
        return ei.value.status
    src, dst = CASES["sequence 2 -> 4"]
    # a destination tensor the source does not have
    other = pack([[(9, 0, 2, (4, 64, 48), (0, 0, 0), (4, 64, 48), (0, 1, 2))]])
    assert st(lambda: plan_of(src, other)) == B.TPX_ERR_INVALID_ARG
    # the source covers only half of the tensor
    assert st(lambda: plan_of(src[:1], dst)) == B.TPX_ERR_INVALID_ARG
    # source sub-tensors overlap without being equal
    bad = pack([[(0, 0, 2, (4, 64, 48), (0, 0, 0), (4, 40, 48), (0, 1, 2))], [(0, 0, 2, (4, 64, 48), (0, 32, 0), (4, 64, 48), (0, 1, 2))]])
    assert st(lambda: plan_of(bad, dst)) == B.TPX_ERR_INVALID_ARG
    # two sub-tensors overlap inside one rank buffer
    e = src[0][0][0]
    clash = [([e, e._replace(tensor_id=1)], src[0][1])]
    assert st(lambda: plan_of(clash, clash)) == B.TPX_ERR_INVALID_ARG
    # a lost rank without a replica
    assert st(lambda: plan_of(src, dst, src_alive=[1, 0])) == B.TPX_ERR_UNRECOVERABLE
    # malformed entries
    assert st(lambda: plan_of([([e._replace(perm=(0, 0, 2))], src[0][1])], dst)) == B.TPX_ERR_INVALID_ARG
    assert st(lambda: plan_of([([e._replace(hi=(4, 99, 48))], src[0][1])], dst)) == B.TPX_ERR_INVALID_ARG
    assert st(lambda: plan_of([([e._replace(elem_bytes=3)], src[0][1])], dst)) == B.TPX_ERR_INVALID_ARG


def test_lost_rank_with_replica_is_recovered():
    src = replicated(2, sequence(2))           # ranks 0,1 and their copies 2,3
    dst = sequence(4)
    a = H.np_bufs(src_buffers(src, 3))
    want = oreshard.reshard_ptc(src, dst, a)
    plan = plan_of(src, dst, src_alive=[0, 1, 1, 0])
    assert {b.src_rank for b in plan.boxes()} == {1, 2}
    a[0][:] = 0xEE
    a[3][:] = 0xEE
    got = [np.full(n, H.POISON, dtype=np.uint8) for _, n in dst]
    host_exec.run_boxes(plan, a, got)
    assert all(np.array_equal(g, w) for g, w in zip(got, want))


def test_range_queries_gather_sub_tensors_from_their_holders():
    """Section 5.2's range query: arbitrary boxes of tensors of a (T,P,D) = (3,2,1) job gathered into one dense buffer;
    expected = the same slice of the full tensor the oracle reassembles."""
    from oracle import spec
    from tests.test_planner import SMALL, SMALL_MIX
    model, par = SMALL, spec.Parallel(3, 2, 1, w_transposed=1)
    src = [spec.rank_manifest(model, par, r) for r in range(par.n_ranks)]
    bufs = H.np_bufs(H.make_src_bufs(model, par, 8, SMALL_MIX))
    lay = oreshard.Layout(manifests=src)
    dense = spec.tensor_id(spec.DENSE_W, 1)
    qkv = spec.tensor_id(spec.QKV_W, 3)
    queries = [(dense, 0, (0, 2), (24, 4)),            # weight[:, 2:4] of a row-parallel tensor: columns of one shard
               (dense, 1, (5, 6), (9, 20)),            # a box that spans all three shards
               (qkv, 1, (3, 1, 0, 7), (10, 3, 2, 19)),  # heads 3..9, K and V, both rows of each head
               (0, 0, (10, 0), (30, 24))]              # embedding rows from two vocabulary shards
    plan = tpx.tpx_plan_query([[H.desc_of(e) for e in ent] for ent, _ in src], queries, src_bytes=[n for _, n in src])
    assert plan.num_buffers(1) == 1
    got = [np.full(plan.buffer_bytes(1, 0), H.POISON, dtype=np.uint8)]
    host_exec.run_tiles(plan, bufs, got)
    for q, e in zip(queries, plan.manifest(1, 0)):
        full = oreshard.full_tensor(None, None, lay, q[0], q[1], lambda r, off, n: bufs[r][off:off + n])
        want = np.ascontiguousarray(full[tuple(slice(l, h) for l, h in zip(q[2], q[3]))])
        have = got[0][e.offset:e.offset + want.nbytes].view(want.dtype).reshape(want.shape)
        assert np.array_equal(have, want), q
    with pytest.raises(tpx.TpxError):
        tpx.tpx_plan_query([[H.desc_of(e) for e in ent] for ent, _ in src], [(9999, 0, (0,), (1,))])


def test_only_wanted_destination_ranks_are_built():
    src, dst = sequence(2), sequence(4)
    a = H.np_bufs(src_buffers(src, 3))
    want = oreshard.reshard_ptc(src, dst, a)
    plan = plan_of(src, dst, dst_alive=[0, 1, 0, 1])
    assert {b.dst_rank for b in plan.boxes()} == {1, 3}
    got = [np.full(n, H.POISON, dtype=np.uint8) for _, n in dst]
    host_exec.run_tiles(plan, a, got)
    assert np.array_equal(got[1], want[1]) and np.array_equal(got[3], want[3])
    assert (got[0] == H.POISON).all() and (got[2] == H.POISON).all()
    assert plan.stats()["bytes_written"] == sum(H.desc_of(e).nbytes for r in (1, 3) for e in dst[r][0])


@pytest.mark.gpu
@pytest.mark.parametrize("name", list(CASES))
def test_generic_gpu_matches_oracle(cuda, name):
    from tests import gpu_util as G
    print("case", name, flush=True)
    src, dst = CASES[name]
    a = src_buffers(src, 9)
    want = oreshard.reshard_ptc(src, dst, H.np_bufs(a))
    plan = plan_of(src, dst, opts=dict(tile_bytes=8192))
    got, _ = G.execute(plan, [x.cuda() for x in a])
    torch.cuda.synchronize()
    for r in range(len(dst)):
        assert np.array_equal(got[r].cpu().numpy(), want[r]), r


@pytest.mark.gpu
def test_range_queries_and_json_collection_through_the_kernel(cuda):
    """Section 5.2's range queries on a (3,2,1) job with transposed storage, and section 5.1's JSON-described collection,
    executed by the HIP kernel; expected values from the oracle (full_tensor slices, reshard_ptc)."""
    import json
    from oracle import spec as ospec
    from paper_2312_05181_amd import ptc_json
    from tests import gpu_util as G
    from tests.test_planner import SMALL, SMALL_MIX
    model, par = SMALL, ospec.Parallel(3, 2, 1, w_transposed=1)
    src = [ospec.rank_manifest(model, par, r) for r in range(par.n_ranks)]
    cpu = H.make_src_bufs(model, par, 8, SMALL_MIX)
    bufs = H.np_bufs(cpu)
    lay = oreshard.Layout(manifests=src)
    dense, qkv = ospec.tensor_id(ospec.DENSE_W, 1), ospec.tensor_id(ospec.QKV_W, 3)
    queries = [(dense, 0, (0, 2), (24, 4)), (dense, 1, (5, 6), (9, 20)), (qkv, 1, (3, 1, 0, 7), (10, 3, 2, 19)),
               (0, 0, (10, 0), (30, 24)), (ospec.tensor_id(ospec.FC1_B, 2), 0, (7,), (41,))]
    plan = tpx.tpx_plan_query([[H.desc_of(e) for e in ent] for ent, _ in src], queries, src_bytes=[n for _, n in src])
    got, _ = G.execute(plan, [x.cuda() for x in cpu])
    torch.cuda.synchronize()
    out = got[0].cpu().numpy()
    covered = np.zeros(out.size, dtype=bool)
    for q, e in zip(queries, plan.manifest(1, 0)):
        full = oreshard.full_tensor(None, None, lay, q[0], q[1], lambda r, off, n: bufs[r][off:off + n])
        want = np.ascontiguousarray(full[tuple(slice(l, h) for l, h in zip(q[2], q[3]))])
        assert e.offset % 256 == 0 and e.nbytes == want.nbytes
        assert np.array_equal(out[e.offset:e.offset + want.nbytes].view(want.dtype).reshape(want.shape), want), q
        covered[e.offset:e.offset + want.nbytes] = True
    assert (out[~covered] == H.POISON).all()

    def gpu(t, T):
        return {"mlp": {"fc1": {"weight": {"full_shape": [640, 96], "offset": [640 // T * t, 0], "shape": [640 // T, 96], "dtype": "bfloat16"},
                                "bias": {"full_shape": [640], "offset": [640 // T * t], "shape": [640 // T], "dtype": "float32"}},
                        "fc2": {"weight": {"full_shape": [96, 640], "offset": [0, 640 // T * t], "shape": [96, 640 // T], "dtype": "bfloat16",
                                           "perm": [1, 0] if T == 4 else [0, 1]}}},
                "ln": {"weight": {"full_shape": [96], "dtype": "float32"}}}
    src_m, dst_m, _ = ptc_json.manifests_from_json(json.dumps([gpu(t, 2) for t in range(2)]), json.dumps([gpu(t, 4) for t in range(4)]))
    plan = tpx.tpx_plan_ptc(src_m, dst_m, opts=dict(tile_bytes=4096))
    src, dst = _collection_of(plan, 0), _collection_of(plan, 1)
    a = []
    for entries, n in src:
        buf = torch.full((n,), H.SRC_GAP, dtype=torch.uint8)
        for e in entries:
            d = H.desc_of(e)
            synth.fill_buffer(buf, [d], 1, ((d.elem_bytes, "index"),))
        a.append(buf)
    want = oreshard.reshard_ptc(src, dst, H.np_bufs(a))
    got, _ = G.execute(plan, [x.cuda() for x in a])
    torch.cuda.synchronize()
    assert all(np.array_equal(g.cpu().numpy(), w) for g, w in zip(got, want))


def _collection_of(plan, side):
    """[(entries, buffer bytes)] per rank as the oracle takes them, read back from a plan's manifests."""
    out = []
    for r in range(plan.num_buffers(side)):
        ent = [spec.Entry(e.tensor_id, e.kind, e.elem_bytes, e.offset, tuple(e.full_shape[:e.ndim]), tuple(e.lo[:e.ndim]),
                          tuple(e.hi[:e.ndim]), tuple(e.perm[:e.ndim]), e.name, e.layer) for e in plan.manifest(side, r)]
        out.append((ent, plan.buffer_bytes(side, r)))
    return out


BIG = {
    # expert parallelism at the size of a small mixture-of-experts layer stack: 8 or 16 experts of two 4096 x 1024 matrices,
    # four state kinds (14 bytes per parameter): 0.9 and 1.9 GB; sequence parallelism on a [8, 4096, 4096] bf16 activation: 268 MB;
    # a 2-D grid of a [8192, 6144] tensor (bf16 + fp32)
    "experts ep8 -> ep4 x tp2": lambda: (experts(8, n_experts=8, h=1024, f=4096), experts(8, tp=2, n_experts=8, h=1024, f=4096)),
    "experts ep4 x tp4 -> ep16": lambda: (experts(16, tp=4, n_experts=16, h=1024, f=4096), experts(16, n_experts=16, h=1024, f=4096)),
    "sequence 8 -> 6": lambda: (sequence(8, batch=8, seq=4096, hidden=4096), sequence(6, batch=8, seq=4096, hidden=4096)),
    "2-D grid 4x2 -> 2x6": lambda: (grid2d(4, 2, shape=(8192, 6144)), grid2d(2, 6, shape=(8192, 6144))),
}


@pytest.mark.gpu
@pytest.mark.parametrize("name", list(BIG))
def test_generic_collections_at_scale_gpu(cuda, name):
    """Expert-, sequence- and grid-parallel collections large enough for the default launch shape (64 KiB tiles, merge tiles,
    thousands of workgroups): every destination buffer equals the generic oracle's, byte for byte, and the value function."""
    from tests import gpu_util as G
    print("case", name, flush=True)
    src, dst = BIG[name]()
    a = src_buffers(src, 19)
    want = oreshard.reshard_ptc(src, dst, H.np_bufs(a), threads=8)
    plan = plan_of(src, dst)
    assert plan.num_tiles() > 2000
    got, _ = G.execute(plan, [x.cuda() for x in a])
    torch.cuda.synchronize()
    exact = closed_form(dst, 19)
    for r in range(len(dst)):
        have = got[r].cpu()
        assert np.array_equal(have.numpy(), want[r]), r
        assert torch.equal(have, exact[r]), r


@pytest.mark.gpu
@pytest.mark.parametrize("eb", [1, 2, 4, 8])
def test_transposing_blocks_of_every_element_size_gpu(cuda, eb):
    """A [1100, 1048] tensor stored row-major in two row halves and wanted column-major in three column thirds, the last third
    twice (replicas: one multicast move): 2-, 4- and 8-byte elements go through the one-shot 64 KiB transposing blocks where a
    block is full and aligned and through the general path at the ragged edges, 1-byte elements through the general path only."""
    from tests import gpu_util as G
    shape = (1100, 1048)
    src = pack([[(0, 0, eb, shape, (a, 0), (b, shape[1]), (0, 1))] for a, b in ((0, 512), (512, 1100))])
    cols = ((0, 352), (352, 704), (704, 1048), (704, 1048))
    dst = pack([[(0, 0, eb, shape, (0, c), (shape[0], d), (1, 0))] for c, d in cols])
    mix = ((eb, "index"),)
    a = []
    for entries, n in src:
        b = torch.full((n,), H.SRC_GAP, dtype=torch.uint8)
        synth.fill_buffer(b, [H.desc_of(e) for e in entries], 29, mix)
        a.append(b)
    want = oreshard.reshard_ptc(src, dst, H.np_bufs(a))
    plan = plan_of(src, dst)
    tiles = plan.tiles()
    assert {t.kind for t in tiles} == {B.TILE_TRANSPOSE} and any(t.n_dst == 2 for t in tiles)
    full = [t for t in tiles if t.nrows * t.run_units * eb == 65536]
    assert bool(full) == (eb > 1)
    got, _ = G.execute(plan, [x.cuda() for x in a])
    torch.cuda.synchronize()
    for r in range(len(dst)):
        assert np.array_equal(got[r].cpu().numpy(), want[r]), r


def _long_run_pair(n, eb, kind):
    """One rank on either side; a small tensor changes place with a long one, so the long one moves as a single contiguous run
    between different offsets."""
    small = (1, 1, 4, (64,), (0,), (64,), (0,))
    big = (0, kind, eb, (n,), (0,), (n,), (0,))
    return pack([[small, big]]), pack([[big, small]])


def test_contiguous_run_beyond_32_bit_unit_counts():
    """A single contiguous move of 40 GiB + 1 bytes (so 1-byte units, twenty times what a 32-bit count of units holds) is planned
    as consecutive tiles that cover it exactly once, source and destination advancing together."""
    import ctypes as C
    n = 40 * (1 << 30) + 1
    src, dst = _long_run_pair(n, 1, 0)
    plan = plan_of(src, dst)
    st = plan.stats()
    assert st["bytes_read"] == st["bytes_written"] == n + 256 and st["n_boxes"] == 2
    tile, pos, seen_small = B.tpx_tile(), 0, 0
    for i in range(plan.num_tiles()):
        assert B._lib.tpx_get_tile(plan._h, i, C.byref(tile)) == 0
        nbytes = tile.nrows * (tile.run_units << tile.unit_log2)
        if tile.src_off == 0:                      # the small tensor: first on the source, last on the destination
            assert tile.dst_off == dst[0][0][1].offset and nbytes == 256
            seen_small += 1
            continue
        assert tile.nrows == 1 and tile.src_off == 256 + pos and tile.dst_off == pos and 0 < nbytes <= 65536, i
        pos += nbytes
    assert pos == n and seen_small == 1


def test_more_rows_than_a_32_bit_count():
    """A [5*10^9, 32] byte tensor held whole by one rank, cut by columns for two ranks: each destination is one move of 5*10^9
    rows of 16 bytes (pitch 32 on the source, 16 on the destination); the tiles cover every row once, in order."""
    import ctypes as C
    n = 5 * 10 ** 9
    src = pack([[(0, 0, 1, (n, 32), (0, 0), (n, 32), (0, 1))]])
    dst = pack([[(0, 0, 1, (n, 32), (0, 16 * j), (n, 16 * j + 16), (0, 1))] for j in range(2)])
    plan = plan_of(src, dst, opts=dict(tile_bytes=1 << 20))
    assert plan.stats()["bytes_written"] == 32 * n
    tile, rows = B.tpx_tile(), [0, 0]
    for i in range(plan.num_tiles()):
        assert B._lib.tpx_get_tile(plan._h, i, C.byref(tile)) == 0
        j = tile.dst_rank
        assert (tile.src_off, tile.dst_off, tile.src_pitch, tile.dst_pitch) == (32 * rows[j] + 16 * j, 16 * rows[j], 32, 16), i
        assert tile.run_units << tile.unit_log2 == 16 and 0 < tile.nrows <= 65536
        rows[j] += tile.nrows
    assert rows == [n, n]


@pytest.mark.gpu
def test_contiguous_run_beyond_32_bit_unit_counts_gpu(cuda):
    """2^31 + 12,345 two-byte elements in one move: an odd count, so the unit is 2 bytes and the run exceeds 2^31 units; the
    kernel's result equals the generic oracle's and the value function, byte for byte."""
    from tests import gpu_util as G
    n = (1 << 31) + 12345
    src, dst = _long_run_pair(n, 2, 0)
    plan = plan_of(src, dst)
    assert {t.unit_log2 for t in (plan.tiles()[0], plan.tiles()[-2])} == {1}
    a = G.alloc(src[0][1], H.SRC_GAP)
    synth.fill_buffer(a, [H.desc_of(e) for e in src[0][0]], 23, MIX)
    got, _ = G.execute(plan, [a])
    torch.cuda.synchronize()
    assert synth.count_mismatch(got[0], [H.desc_of(e) for e in dst[0][0]], 23, MIX) == 0
    want = oreshard.reshard_ptc(src, dst, [a.cpu().numpy()], threads=8)
    assert np.array_equal(got[0].cpu().numpy(), want[0])


def test_json_configuration_importer():
    """Two per-GPU JSON documents (paper section 5.1) describing a two-matrix model under 2-way tensor
    parallelism and under 1 GPU; the imported collections re-partition like the oracle says."""
    import json
    from paper_2312_05181_amd import ptc_json

    def gpu(t, T):
        return {"mlp": {"fc1": {"weight": {"full_shape": [64, 32], "offset": [64 // T * t, 0], "shape": [64 // T, 32], "dtype": "bfloat16"},
                                "bias": {"full_shape": [64], "offset": [64 // T * t], "shape": [64 // T], "dtype": "float32"}},
                        "fc2": {"weight": {"full_shape": [32, 64], "offset": [0, 64 // T * t], "shape": [32, 64 // T], "dtype": "bfloat16"}}},
                "ln": {"weight": {"full_shape": [32], "dtype": "float32"}}}
    src_m, dst_m, names = ptc_json.manifests_from_json(json.dumps([gpu(0, 2), gpu(1, 2)]), json.dumps([gpu(0, 1)]))
    assert names == ["/ln/weight", "/mlp/fc1/bias", "/mlp/fc1/weight", "/mlp/fc2/weight"]
    plan = tpx.tpx_plan_ptc(src_m, dst_m)           # the library places every block in its rank buffer
    src, dst = _collection_of(plan, 0), _collection_of(plan, 1)
    dst_b = [n for _, n in dst]
    assert [e.offset for e in src[0][0]] == [0, 2048, 2304, 4352] and src[0][1] == 4608     # document order, 256-byte aligned
    mix = ((4, "index"),)
    a = []
    for entries, n in src:
        buf = torch.full((n,), H.SRC_GAP, dtype=torch.uint8)
        for e in entries:
            d = H.desc_of(e)
            synth.fill_buffer(buf, [d], 1, ((d.elem_bytes, "index"),))
        a.append(buf.numpy())
    want = oreshard.reshard_ptc(src, dst, a)
    got = [np.full(n, H.POISON, dtype=np.uint8) for n in dst_b]
    host_exec.run_tiles(plan, a, got)
    assert all(np.array_equal(g, w) for g, w in zip(got, want))


def _fig5_collection():
    """The collection of paper figure 5, built from the fixture: data tensors t1, t2 (a sample batch each) and
    model tensors t3, t4 (sliced in two along axis 0), one unified collection of tensors."""
    import os
    shapes = {"t1": (4, 16), "t2": (4, 16), "t3": (8, 6), "t4": (10, 4)}
    ids = {"t1": 1, "t2": 2, "t3": 3, "t4": 4}
    ranks = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "fig5_tp2_dp2.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if not line:
                continue
            per = []
            data = line[1]
            per.append((ids[data], 0, 4, shapes[data], (0, 0), shapes[data], (0, 1)))
            for sub in line[2:]:
                name, part = sub.split("^")
                full = shapes[name]
                a, b = even(full[0], 2, int(part) - 1)
                per.append((ids[name], 0, 4, full, (a, 0), (b, full[1]), (0, 1)))
            ranks.append(per)
    return pack(ranks)


def test_fig5_unified_collection_reconfigures():
    """Figure 5's collection (data and model state as one tensor collection) against this library's rank
    order, and its reconfiguration to data parallelism only (4 GPUs, full model each, half a batch each)."""
    src = _fig5_collection()
    assert len(src) == 4
    # alpha of this library: rank = t + T*d reproduces the figure's R1..R4 (cross product of data and model parts)
    for r, (entries, _) in enumerate(src):
        t, d = r % 2, r // 2
        assert entries[0].tensor_id == 1 + d                                  # data sub-collection of replica d
        assert all(e.lo[0] == even(e.full_shape[0], 2, t)[0] for e in entries[1:])   # model part t
    plan_same = plan_of(src, src)
    assert plan_same.stats()["bytes_cross_rank"] == 0
    # new configuration: no tensor parallelism, 4 data-parallel replicas, each data tensor cut in two sample halves
    ranks = []
    for r in range(4):
        data_id, half = 1 + r // 2, r % 2
        per = [(data_id, 0, 4, (4, 16), (2 * half, 0), (2 * half + 2, 16), (0, 1))]
        per += [(3, 0, 4, (8, 6), (0, 0), (8, 6), (0, 1)), (4, 0, 4, (10, 4), (0, 0), (10, 4), (0, 1))]
        ranks.append(per)
    dst = pack(ranks)
    mix = ((4, "index"),)
    a = []
    for entries, n in src:
        b = torch.full((n,), H.SRC_GAP, dtype=torch.uint8)
        synth.fill_buffer(b, [H.desc_of(e) for e in entries], 2, mix)
        a.append(b.numpy())
    want = oreshard.reshard_ptc(src, dst, a)
    plan = plan_of(src, dst)
    got = [np.full(n, H.POISON, dtype=np.uint8) for _, n in dst]
    host_exec.run_tiles(plan, a, got)
    assert all(np.array_equal(g, w) for g, w in zip(got, want))
    # every model tensor is merged from its two halves; every data half is taken from the GPU's own copy of the batch
    assert {(b.src_rank, b.dst_rank) for b in plan.boxes() if b.tensor_id in (1, 2)} == {(0, 0), (1, 1), (2, 2), (3, 3)}
    assert {b.src_rank for b in plan.boxes() if b.tensor_id == 3 and b.dst_rank == 0} == {0, 1}
