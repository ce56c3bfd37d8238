"""Pins of the CPU oracle against things other than itself: closed forms,
hand-written fixtures, the mathematics of tensor parallelism, a library routine
(np.split / np.concatenate), and invariants.  No GPU and no product code."""
import itertools
import os

import numpy as np
import pytest
import torch

import synth
from oracle import reshard as oreshard
from oracle import spec
from oracle.spec import Model, Parallel
from tests import helpers as H

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------
# closed forms
# --------------------------------------------------------------------------
@pytest.mark.parametrize("model,T,expect", [
    (H.TINY, 1, 2_104_320),
    (H.GPT_1_3B, 1, 1_313_722_368),
    (H.GPT_2_7B, 1, 2_649_052_160),
    (H.GPT_6_7B, 1, 6_654_402_560),
    (H.GPT_ODD, 3, 2_876_553_216),
])
def test_parameter_counts(model, T, expect):
    # per layer 12 h^2 + 13 h (ffn = 4 h); plus (V_pad + S) h + 2 h
    h = model.hidden
    assert model.n_layers * (12 * h * h + 13 * h) + (spec.vocab_padded(model, T) + model.max_pos) * h + 2 * h == expect
    assert spec.n_params(model, T) == expect


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_manifest_bytes_match_closed_form(cfg):
    """Sum over ranks of stored bytes = bytes/param x (split params + T x replicated params) x D."""
    model, src, dst, _, _ = H.CONFIGS[cfg]
    bpp = sum(model.state_elem_bytes)
    h = model.hidden
    for par in (src, dst):
        repl = model.n_layers * 6 * h + model.max_pos * h + 2 * h     # per layer: 4 LayerNorm vectors + 2 row-parallel biases
        split = spec.n_params(model, par.T) - repl
        assert oreshard.state_bytes(model, par) == bpp * (split + par.T * repl) * par.D


def test_vocab_padding_values():
    assert spec.vocab_padded(H.GPT_ODD, 3) == 50304
    assert spec.vocab_padded(H.GPT_ODD, 4) == 50688
    assert spec.vocab_padded(H.GPT_6_7B, 8) == 50304
    with pytest.raises(ValueError):
        spec.vocab_padded(Model(2, 8, 2, 16, 1001), 2)


# --------------------------------------------------------------------------
# hand-written fixtures
# --------------------------------------------------------------------------
def _load_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append([int(x) for x in line.split()])
    return rows


def test_fig6_two_way_to_three_way_golden():
    """Paper figure 6: a tensor sliced in two is re-sliced in three; the middle third
    is merged from the tail of the first half and the head of the second half."""
    rows = _load_golden("fig6_tp2_to_tp3.txt")
    src_shards, dst_shards = rows[:2], rows[2:5]
    # a model whose mlp.dense_h_to_4h.bias (axis-0 split, 1-D, ffn elements) is the tensor of the figure
    model = Model(n_layers=1, hidden=6, n_heads=6, ffn=12, vocab_true=6, max_pos=1, state_elem_bytes=(4,))
    src, dst = Parallel(2, 1, 1), Parallel(3, 1, 1)
    mix = ((4, "index"),)
    bufs = H.np_bufs(H.make_src_bufs(model, src, 0, mix))
    tid = spec.tensor_id(spec.FC1_B, 0)
    for r in range(2):
        e = [e for e in spec.rank_manifest(model, src, r)[0] if e.tensor_id == tid][0]
        bufs[r][e.offset:e.offset + 24] = np.array(src_shards[r], dtype=np.uint32).view(np.uint8)
    out = oreshard.reshard(model, src, dst, bufs)
    for r in range(3):
        e = [e for e in spec.rank_manifest(model, dst, r)[0] if e.tensor_id == tid][0]
        got = out[r][e.offset:e.offset + 16].view(np.uint32)
        assert got.tolist() == dst_shards[r]


def test_qkv_head_interleave_golden():
    """Fused QKV, 2 heads of dim 1, hidden 2: rows are Q0 K0 V0 Q1 K1 V1 (head-major).
    Two-way tensor parallelism gives rank 0 the rows of head 0 and rank 1 those of head 1;
    the qkv-major layout stores a rank's rows as all Q, then all K, then all V."""
    rows = _load_golden("qkv_interleave.txt")
    full_rows = rows[0:6]            # full [3h, h] weight, head-major
    model = Model(n_layers=1, hidden=2, n_heads=2, ffn=2, vocab_true=2, max_pos=1, state_elem_bytes=(4,))
    one = Parallel(1, 1, 1)
    mix = ((4, "index"),)
    bufs = H.np_bufs(H.make_src_bufs(model, one, 0, mix))
    tid = spec.tensor_id(spec.QKV_W, 0)
    e = [e for e in spec.rank_manifest(model, one, 0)[0] if e.tensor_id == tid][0]
    bufs[0][e.offset:e.offset + 48] = np.array(full_rows, dtype=np.uint32).reshape(-1).view(np.uint8)
    # head-major, T=2
    out = oreshard.reshard(model, one, Parallel(2, 1, 1), bufs)
    for r, want in enumerate((rows[6:9], rows[9:12])):
        e = [e for e in spec.rank_manifest(model, Parallel(2, 1, 1), r)[0] if e.tensor_id == tid][0]
        assert out[r][e.offset:e.offset + 24].view(np.uint32).reshape(3, 2).tolist() == want
    # qkv-major, T=1: Q0 Q1 K0 K1 V0 V1
    qm = Parallel(1, 1, 1, qkv_layout=1)
    out = oreshard.reshard(model, one, qm, bufs)
    e = [e for e in spec.rank_manifest(model, qm, 0)[0] if e.tensor_id == tid][0]
    assert out[0][e.offset:e.offset + 48].view(np.uint32).reshape(6, 2).tolist() == rows[12:18]


# --------------------------------------------------------------------------
# library routine: shards are numpy's equal split of the full tensor
# --------------------------------------------------------------------------
SMALL = Model(n_layers=4, hidden=24, n_heads=12, ffn=48, vocab_true=36, max_pos=5, state_elem_bytes=(4, 2))
SMALL_MIX = ((4, "u11"), (2, "index"))


def _full_from_value_function(model, name, layer, kind, seed, mix, T):
    full_shape, _, _ = spec.canonical(model, Parallel(T, 1, 1), name)
    d = synth.ShardDesc(spec.tensor_id(name, layer), kind, mix[kind][0], 0, full_shape,
                        (0,) * len(full_shape), full_shape, tuple(range(len(full_shape))))
    v = synth.block_values(seed, d, mix[kind][1], "cpu")
    return v.view(torch.int32 if mix[kind][0] == 4 else torch.int16).numpy()


@pytest.mark.parametrize("T", [1, 2, 3, 4, 6])
def test_shards_are_numpy_split_of_full(T):
    """concat(shards along the split axis) == full tensor (spec invariant), using
    np.split as the independent slicer.  Head-major QKV [3h, h] splits as plain row blocks."""
    model, mix, seed = SMALL, SMALL_MIX, 11
    par = Parallel(T, 2, 1)
    bufs = H.np_bufs(H.make_src_bufs(model, par, seed, mix))
    axis_of = {spec.WORD_EMB: 0, spec.QKV_W: 0, spec.QKV_B: 0, spec.DENSE_W: 1, spec.FC1_W: 0,
               spec.FC1_B: 0, spec.FC2_W: 1}
    for rank in range(par.n_ranks):
        t, p, d = spec.coords_of(par, rank)
        for e in spec.rank_manifest(model, par, rank)[0]:
            full = _full_from_value_function(model, e.name, e.layer, e.kind, seed, mix, T)
            if e.name in (spec.QKV_W, spec.QKV_B):     # plain [3h, h] / [3h] view of the fused tensor
                full = full.reshape((3 * model.hidden,) + full.shape[3:])
            want = np.split(full, T, axis=axis_of[e.name])[t] if e.name in axis_of else full
            dt = np.int32 if e.elem_bytes == 4 else np.int16
            got = bufs[rank][e.offset:e.offset + want.nbytes].view(dt).reshape(want.shape)
            assert np.array_equal(got, want), (rank, spec.NAMES[e.name][0])


@pytest.mark.parametrize("D", [2, 3, 4, 7])
@pytest.mark.parametrize("tags", [dict(), dict(qkv_layout=1), dict(w_transposed=1)])
def test_sharded_kinds_partition_each_share(D, tags):
    """Sharded data parallelism: the chunks the D replicas keep of a tensor, concatenated in replica order
    along the outermost stored axis, are exactly the block a replica of the unsharded configuration holds;
    chunk d has min(c, max(0, n - d*c)) rows with c = ceil(n / D); kinds that are not sharded are untouched."""
    model, mix, seed = SMALL, SMALL_MIX, 13
    whole, cut = Parallel(2, 2, 1, **tags), Parallel(2, 2, D, shard_kinds=2, **tags)
    ref = H.np_bufs(H.make_src_bufs(model, whole, seed, mix))
    got = H.np_bufs(H.make_src_bufs(model, cut, seed, mix))
    total = 0
    for t in range(2):
        for p in range(2):
            for e in spec.rank_manifest(model, whole, spec.rank_of(whole, t, p, 0))[0]:
                stored = tuple(e.hi[a] - e.lo[a] for a in e.perm)
                want = ref[spec.rank_of(whole, t, p, 0)][e.offset:e.offset + int(np.prod(stored)) * e.elem_bytes]
                chunks = []
                for d in range(D):
                    r = spec.rank_of(cut, t, p, d)
                    mine = [x for x in spec.rank_manifest(model, cut, r)[0] if (x.tensor_id, x.kind) == (e.tensor_id, e.kind)]
                    if e.kind == 0:                    # replicated as before
                        assert len(mine) == 1 and (mine[0].lo, mine[0].hi) == (e.lo, e.hi)
                        x = mine[0]
                        assert np.array_equal(got[r][x.offset:x.offset + want.nbytes], want)
                        continue
                    n = stored[0]
                    c = -(-n // D)
                    rows = min(c, max(0, n - d * c))
                    assert len(mine) == (1 if rows else 0), (d, n)
                    if rows:
                        x = mine[0]
                        assert x.hi[x.perm[0]] - x.lo[x.perm[0]] == rows
                        nbytes = rows * int(np.prod(stored[1:])) * x.elem_bytes
                        chunks.append(got[r][x.offset:x.offset + nbytes])
                        total += nbytes
                if e.kind == 1:
                    assert np.array_equal(np.concatenate(chunks), want), (t, p, spec.NAMES[e.name][0])
    # closed form: the sharded kind is stored once, not D times
    one = Parallel(2, 2, 1)
    per_kind = [sum(int(np.prod([h - l for l, h in zip(e.lo, e.hi)])) * e.elem_bytes
                    for r in range(one.n_ranks) for e in spec.rank_manifest(model, one, r)[0] if e.kind == k) for k in (0, 1)]
    assert total == per_kind[1]
    assert oreshard.state_bytes(model, cut) == D * per_kind[0] + per_kind[1]


# --------------------------------------------------------------------------
# mathematics: a tensor-parallel layer built from the shards computes the same
# function as the unsharded layer
# --------------------------------------------------------------------------
def _gelu(x):
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def _layer_forward(x, ids, blocks, model, par):
    """Forward of embedding + one transformer layer (no LayerNorm affine shortcuts taken)
    from the stored blocks of a T-way tensor-parallel job.  blocks[t][name] is rank t's
    stored block as float64, in its storage order."""
    T, h, a, dh = par.T, model.hidden, model.n_heads, model.head_dim
    al = a // T
    vp = spec.vocab_padded(model, T) // T

    def lin(w_stored, inp):        # y = inp @ W^T with W = [out, in]; transposed storage holds W^T
        return inp @ (w_stored if par.w_transposed else w_stored.T)

    emb = np.zeros((len(ids), h))
    for t in range(T):
        local = ids - t * vp
        ok = (local >= 0) & (local < vp)
        emb[ok] += blocks[t][spec.WORD_EMB][local[ok]]
    x = x + emb + blocks[0][spec.POS_EMB][:len(ids)]

    def ln(v, w, b):
        mu = v.mean(-1, keepdims=True)
        return (v - mu) / np.sqrt(v.var(-1, keepdims=True) + 1e-5) * w + b

    y = ln(x, blocks[0][spec.LN1_W], blocks[0][spec.LN1_B])
    attn_out = np.zeros_like(x)
    for t in range(T):
        w = blocks[t][spec.QKV_W]
        bq = blocks[t][spec.QKV_B]
        if par.w_transposed:                       # stored [h, out...]: bring `in` last
            w = np.moveaxis(w, 0, -1)
        if par.qkv_layout == 0:                    # [al, 3, dh, h]
            wq, wk, wv = w[:, 0], w[:, 1], w[:, 2]
            bq_, bk_, bv_ = bq[:, 0], bq[:, 1], bq[:, 2]
        else:                                      # [3, al, dh, h]
            wq, wk, wv = w[0], w[1], w[2]
            bq_, bk_, bv_ = bq[0], bq[1], bq[2]
        ctx = []
        for i in range(al):
            q = y @ wq[i].T + bq_[i]
            k = y @ wk[i].T + bk_[i]
            v = y @ wv[i].T + bv_[i]
            s = q @ k.T / np.sqrt(dh)
            s = np.where(np.tril(np.ones_like(s)) > 0, s, -1e30)
            pr = np.exp(s - s.max(-1, keepdims=True))
            pr /= pr.sum(-1, keepdims=True)
            ctx.append(pr @ v)
        ctx = np.concatenate(ctx, axis=-1)                      # [seq, h/T]
        attn_out += lin(blocks[t][spec.DENSE_W], ctx)           # row-parallel: partial sums
    x = x + attn_out + blocks[0][spec.DENSE_B]
    y = ln(x, blocks[0][spec.LN2_W], blocks[0][spec.LN2_B])
    mlp = np.zeros_like(x)
    for t in range(T):
        hmid = _gelu(lin(blocks[t][spec.FC1_W], y) + blocks[t][spec.FC1_B])
        mlp += lin(blocks[t][spec.FC2_W], hmid)
    x = x + mlp + blocks[0][spec.FC2_B]
    return ln(x, blocks[0][spec.LNF_W], blocks[0][spec.LNF_B])


def _blocks_of(model, par, bufs):
    out = []
    for t in range(par.T):
        entries = spec.rank_manifest(model, par, spec.rank_of(par, t, 0, 0))[0]
        b = {}
        for e in entries:
            shp = tuple(e.hi[a] - e.lo[a] for a in e.perm)
            n = int(np.prod(shp)) * 8
            b[e.name] = bufs[spec.rank_of(par, t, 0, 0)][e.offset:e.offset + n].view(np.float64).reshape(shp)
        out.append(b)
    return out


@pytest.mark.parametrize("dst", [
    Parallel(2, 1, 1), Parallel(4, 1, 1), Parallel(3, 1, 1),
    Parallel(2, 1, 1, qkv_layout=1), Parallel(4, 1, 1, qkv_layout=1),
    Parallel(2, 1, 1, w_transposed=1), Parallel(3, 1, 1, qkv_layout=1, w_transposed=1),
])
def test_tensor_parallel_forward_equivalence(dst):
    """Cutting the layer the way sigma says must leave its function unchanged: column-parallel
    QKV by heads and h->4h by rows, row-parallel projections by input columns, vocabulary-split
    embedding.  A wrong split axis, head order or transposition changes the output."""
    rng = np.random.default_rng(5)
    model = Model(n_layers=1, hidden=24, n_heads=12, ffn=36, vocab_true=50, max_pos=7,
                  vocab_divisor=4, state_elem_bytes=(8,))
    one = Parallel(1, 1, 1)
    entries, n = spec.rank_manifest(model, one, 0)
    buf = np.zeros(n, dtype=np.uint8)
    for e in entries:
        cnt = int(np.prod(e.full_shape))
        buf[e.offset:e.offset + cnt * 8] = (rng.standard_normal(cnt) * 0.3).view(np.uint8)
    ids = rng.integers(0, model.vocab_true, size=7)
    x0 = rng.standard_normal((7, model.hidden)) * 0.1
    ref = _layer_forward(x0, ids, _blocks_of(model, one, [buf]), model, one)
    out = oreshard.reshard(model, one, dst, [buf])
    got = _layer_forward(x0, ids, _blocks_of(model, dst, out), model, dst)
    assert np.allclose(ref, got, rtol=1e-10, atol=1e-12)
    assert np.abs(ref).max() > 0.1


# --------------------------------------------------------------------------
# closed-form value function and invariants
# --------------------------------------------------------------------------
PAIRS = [
    (Parallel(2, 1, 1), Parallel(4, 2, 1)),
    (Parallel(4, 2, 1), Parallel(2, 4, 1)),
    (Parallel(4, 4, 2), Parallel(2, 4, 1, stage_first_layer=(0, 1, 2, 3, 4))),
    (Parallel(4, 2, 2), Parallel(2, 2, 1, stage_first_layer=(0, 1, 4))),
    (Parallel(6, 1, 1), Parallel(1, 4, 1)),
    (Parallel(3, 1, 1), Parallel(4, 1, 1)),
    (Parallel(2, 2, 1), Parallel(2, 2, 2)),
    (Parallel(2, 1, 1, qkv_layout=1), Parallel(3, 2, 1)),
    (Parallel(2, 1, 1), Parallel(4, 1, 1, qkv_layout=1, w_transposed=1)),
    # state kinds sharded over the data-parallel replicas (bit k of shard_kinds)
    (Parallel(2, 1, 2, shard_kinds=2), Parallel(2, 1, 4, shard_kinds=2)),
    (Parallel(4, 2, 2, shard_kinds=2), Parallel(2, 2, 1)),
    (Parallel(2, 1, 1), Parallel(3, 2, 3, shard_kinds=3)),
    (Parallel(2, 1, 3, shard_kinds=1, qkv_layout=1), Parallel(1, 2, 5, shard_kinds=2, w_transposed=1)),
    # any layer -> stage map: interleaved (virtual) pipeline chunks, and one stage left without layers
    (Parallel(2, 2, 1, layer_stage=(0, 1, 0, 1)), Parallel(3, 2, 1)),
    (Parallel(4, 1, 1), Parallel(2, 3, 2, layer_stage=(2, 0, 0, 2), shard_kinds=2)),
]


@pytest.mark.parametrize("src,dst", PAIRS)
def test_reshard_matches_value_function(src, dst):
    """Every destination byte equals g(seed, tensor, kind, position) evaluated directly."""
    model, mix, seed = SMALL, SMALL_MIX, 21
    out = oreshard.reshard(model, src, dst, H.np_bufs(H.make_src_bufs(model, src, seed, mix)))
    want = H.np_bufs(H.closed_form_dst_bufs(model, src, dst, seed, mix))
    for r, (a, b) in enumerate(zip(out, want)):
        assert np.array_equal(a, b), r


def test_vocab_growth_zero_fills_and_round_trip():
    model = Model(n_layers=2, hidden=12, n_heads=12, ffn=24, vocab_true=50, max_pos=3,
                  vocab_divisor=4, state_elem_bytes=(2, 4))
    mix = ((2, "index"), (4, "u11"))
    a, b = Parallel(3, 1, 1), Parallel(4, 1, 1)          # padded vocab 60 -> 64
    assert (spec.vocab_padded(model, 3), spec.vocab_padded(model, 4)) == (60, 64)
    src = H.np_bufs(H.make_src_bufs(model, a, 3, mix))
    mid = oreshard.reshard(model, a, b, src)
    want = H.np_bufs(H.closed_form_dst_bufs(model, a, b, 3, mix))
    assert all(np.array_equal(x, y) for x, y in zip(mid, want))
    # the last 4 rows of the new embedding are zero in every state kind
    e = [e for e in spec.rank_manifest(model, b, 3)[0] if e.name == spec.WORD_EMB]
    for ent in e:
        blk = mid[3][ent.offset:ent.offset + 16 * 12 * ent.elem_bytes].reshape(16, -1)
        assert not blk[12:].any() and blk[:12].any()
    # growing then shrinking the padding is the identity on tensor bytes
    back = oreshard.reshard(model, b, a, mid)
    for r in range(3):
        descs = [H.desc_of(x) for x in spec.rank_manifest(model, a, r)[0]]
        for d in descs:
            assert np.array_equal(back[r][d.offset:d.offset + d.nbytes], src[r][d.offset:d.offset + d.nbytes])


def _tensor_bytes_equal(model, par, x, y):
    for r in range(par.n_ranks):
        for e in spec.rank_manifest(model, par, r)[0]:
            d = H.desc_of(e)
            if not np.array_equal(x[r][d.offset:d.offset + d.nbytes], y[r][d.offset:d.offset + d.nbytes]):
                return False
    return True


@pytest.mark.parametrize("src,dst", PAIRS)
def test_round_trip_is_identity(src, dst):
    model, mix, seed = SMALL, SMALL_MIX, 31
    a = H.np_bufs(H.make_src_bufs(model, src, seed, mix))
    back = oreshard.reshard(model, dst, src, oreshard.reshard(model, src, dst, a))
    assert _tensor_bytes_equal(model, src, a, back)


def test_composition():
    """A -> B -> C equals A -> C."""
    model, mix, seed = SMALL, SMALL_MIX, 41
    cfgs = [Parallel(2, 1, 1), Parallel(4, 2, 1), Parallel(3, 4, 2, qkv_layout=1), Parallel(6, 1, 1),
            Parallel(1, 2, 1, stage_first_layer=(0, 3, 4))]
    for A, B, C in itertools.permutations(cfgs, 3):
        a = H.np_bufs(H.make_src_bufs(model, A, seed, mix))
        via = oreshard.reshard(model, B, C, oreshard.reshard(model, A, B, a))
        direct = oreshard.reshard(model, A, C, a)
        assert all(np.array_equal(x, y) for x, y in zip(via, direct))


def test_replica_disagreement_is_detected():
    model, mix = SMALL, SMALL_MIX
    src = Parallel(2, 1, 2)
    a = H.np_bufs(H.make_src_bufs(model, src, 1, mix))
    e = spec.rank_manifest(model, src, 2)[0][5]
    a[2][e.offset] ^= 1
    with pytest.raises(AssertionError):
        oreshard.reshard(model, src, Parallel(1, 1, 1), a)


def test_fig5_collection_structure():
    """Paper figure 5: tensor parallelism 2 x data parallelism 2 on four GPUs. Each model tensor
    has two sub-tensors; the four sub-collections are the cross product of sub-tensor index and
    replica; both replicas of a sub-tensor hold the same box."""
    model = SMALL
    par = Parallel(2, 1, 2)
    assert par.n_ranks == 4
    tid = spec.tensor_id(spec.FC1_W, 0)
    boxes = {}
    for r in range(4):
        t, p, d = spec.coords_of(par, r)
        e = [e for e in spec.rank_manifest(model, par, r)[0] if e.tensor_id == tid and e.kind == 0][0]
        boxes[(t, d)] = (e.lo, e.hi)
    assert set(boxes) == {(0, 0), (1, 0), (0, 1), (1, 1)}
    assert boxes[(0, 0)] == boxes[(0, 1)] and boxes[(1, 0)] == boxes[(1, 1)]
    assert boxes[(0, 0)] != boxes[(1, 0)]


# --------------------------------------------------------------------------
# planted mistakes: each pin above must notice a plausible bug in the oracle
# --------------------------------------------------------------------------
def test_pins_catch_a_wrong_split_axis(monkeypatch):
    real = spec.canonical

    def wrong(model, par, name):
        full, axis, perm = real(model, par, name)
        if name == spec.DENSE_W:
            axis = 0                      # row-parallel weight cut along the wrong axis
        return full, axis, perm
    monkeypatch.setattr(spec, "canonical", wrong)
    with pytest.raises((AssertionError, ValueError)):
        test_tensor_parallel_forward_equivalence(Parallel(2, 1, 1))
    with pytest.raises((AssertionError, ValueError)):
        test_shards_are_numpy_split_of_full(2)


def test_pins_catch_a_plain_row_split_of_qkv_major(monkeypatch):
    """Treating a [3, a, d] fused tensor as contiguous row blocks mixes Q, K and V of different ranks."""
    real = spec.canonical

    def wrong(model, par, name):
        full, axis, perm = real(model, par, name)
        if name in (spec.QKV_W, spec.QKV_B) and par.qkv_layout == 1:
            a, three, dh = full[:3]
            full = (three, a, dh) + full[3:]         # split axis 0 is now the q/k/v axis: not by heads
            perm = tuple(range(len(full)))
        return full, axis, perm
    monkeypatch.setattr(spec, "canonical", wrong)
    with pytest.raises((AssertionError, ValueError, IndexError)):
        test_tensor_parallel_forward_equivalence(Parallel(3, 1, 1, qkv_layout=1, w_transposed=0))


def test_layer_stage_map_places_each_layer_once():
    """phi for pipeline parallelism as an arbitrary map: every layer's tensors sit on exactly the named stage (every
    tensor-parallel rank and replica of it), embeddings stay on stage 0 and the final LayerNorm on the last stage;
    a contiguous map is the same configuration as the boundary list that describes it."""
    model = SMALL
    par = Parallel(2, 3, 2, layer_stage=(2, 0, 2, 1))
    for rank in range(par.n_ranks):
        t, p, d = spec.coords_of(par, rank)
        entries, _ = spec.rank_manifest(model, par, rank)
        layers = sorted({e.layer for e in entries if e.layer >= 0})
        assert layers == [l for l in range(4) if par.layer_stage[l] == p]
        names = {e.name for e in entries if e.layer < 0}
        assert names == ({spec.WORD_EMB, spec.POS_EMB} if p == 0 else {spec.LNF_W, spec.LNF_B} if p == 2 else set())
        offs = [e.offset for e in entries]
        assert offs == sorted(offs)
    a = [spec.rank_manifest(model, Parallel(2, 2, 1, layer_stage=(0, 0, 0, 1)), r) for r in range(4)]
    b = [spec.rank_manifest(model, Parallel(2, 2, 1, stage_first_layer=(0, 3, 4)), r) for r in range(4)]
    assert a == b
    for bad in ((0, 1, 2), (0, 1, 3, 0), (0, -1, 0, 0)):
        with pytest.raises(ValueError):
            spec.rank_manifest(model, Parallel(2, 3, 1, layer_stage=bad), 0)


def test_sharded_kind_hand_worked_golden():
    rows = _load_golden("sharded_kind_5rows_3replicas.txt")
    block = np.arange(10, 20).reshape(5, 2)
    for D, want in ((3, rows[0:3]), (4, rows[3:6] + [None])):
        for d in range(D):
            got = spec.replica_range((0, 0), (5, 2), (0, 1), D, d)
            if want[d] is None:
                assert got is None
            else:
                lo, hi = got
                assert block[lo[0]:hi[0], lo[1]:hi[1]].reshape(-1).tolist() == want[d]
    # the outermost *stored* axis is cut: a block stored column-major is cut by columns
    assert spec.replica_range((0, 0), (5, 2), (1, 0), 2, 1) == ((0, 1), (5, 2))


def test_pins_catch_floor_sized_replica_chunks(monkeypatch):
    """Planted mistake: chunks of floor(n / D) rows leave the tail of a sharded tensor with no holder."""
    real = spec.replica_range

    def wrong(lo, hi, perm, D, d):
        ax = perm[0]
        n = hi[ax] - lo[ax]
        c = max(1, n // D)
        a, b = min(n, d * c), min(n, (d + 1) * c)
        if a == b:
            return None
        lo2, hi2 = list(lo), list(hi)
        lo2[ax], hi2[ax] = lo[ax] + a, lo[ax] + b
        return tuple(lo2), tuple(hi2)
    monkeypatch.setattr(spec, "replica_range", wrong)
    with pytest.raises(AssertionError):
        test_sharded_kinds_partition_each_share(7, dict())
    monkeypatch.setattr(spec, "replica_range", real)
    test_sharded_kinds_partition_each_share(7, dict())


def test_pins_catch_a_dropped_paste(monkeypatch):
    real = oreshard._box

    def wrong(lo, hi):
        return tuple(slice(l, max(l, u - 1)) if i == 0 else slice(l, u) for i, (l, u) in enumerate(zip(lo, hi)))
    monkeypatch.setattr(oreshard, "_box", wrong)
    with pytest.raises((AssertionError, ValueError)):
        test_reshard_matches_value_function(*PAIRS[0])


# --------------------------------------------------------------------------
# phi: which stage holds which layer when no map is given; the tied output layer's copy
# --------------------------------------------------------------------------
def _stage_rows(name):
    """rows of "a b | x y | ..." fixtures: ([a, b], [[x, y], ...]) per line."""
    out = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                head, *groups = [[int(x) for x in g.split()] for g in line.split("|")]
                out.append((head, groups))
    return out


def test_even_stage_default_places_the_hand_listed_layers():
    """Without a stage map, stage p of P holds layers [p*L/P, (p+1)*L/P) - on every tensor-parallel rank and
    every replica of it - and nothing of any other layer (hand-written lists, including the 2.7B-shape source)."""
    cases = _stage_rows("even_stages.txt")
    assert len(cases) == 4
    for (L, P), stages in cases:
        assert len(stages) == P
        model = Model(n_layers=L, hidden=8, n_heads=2, ffn=8, vocab_true=8, max_pos=2, state_elem_bytes=(2, 4))
        par = Parallel(2, P, 2)
        for rank in range(par.n_ranks):
            t, p, d = spec.coords_of(par, rank)
            entries, _ = spec.rank_manifest(model, par, rank)
            for kind in range(2):
                layers = [e.layer for e in entries if e.kind == kind and e.layer >= 0]
                assert layers == [l for l in stages[p] for _ in range(spec.N_LAYER_NAMES)], (L, P, rank)
    with pytest.raises(ValueError):          # 4 layers cannot be dealt evenly to 3 stages
        spec.rank_manifest(Model(n_layers=4, hidden=8, n_heads=2, ffn=8, vocab_true=8, max_pos=2), Parallel(1, 3, 1), 0)
    # the 2.7B-shape workload's source configuration itself, (4,4,2): ranks of stage 2 hold layers 16..23
    m3, s3 = H.CONFIGS[3][0], H.CONFIGS[3][1]
    for rank in (spec.rank_of(s3, 0, 2, 0), spec.rank_of(s3, 3, 2, 1)):
        assert sorted({e.layer for e in spec.rank_manifest(m3, s3, rank)[0] if e.layer >= 0}) == cases[1][1][2]


def test_pins_catch_a_wrong_even_stage_default(monkeypatch):
    """Planted mistakes in the default stage map: boundaries rounded the wrong way round, and stages in reverse."""
    real = spec.stage_bounds

    def shifted(model, par):
        b = list(real(model, par))
        if par.stage_first_layer is None and par.P > 1:
            b[1] += 1                      # first stage one layer too long
        return tuple(b)
    monkeypatch.setattr(spec, "stage_bounds", shifted)
    with pytest.raises(AssertionError):
        test_even_stage_default_places_the_hand_listed_layers()
    monkeypatch.setattr(spec, "stage_bounds", real)
    real_tensors = spec.stage_tensors

    def reversed_stages(model, par, p):
        out = real_tensors(model, par, p)
        if par.stage_first_layer is None and par.layer_stage is None:
            glob = [x for x in out if x[1] < 0]
            other = [x for x in real_tensors(model, par, par.P - 1 - p) if x[1] >= 0]
            out = [g for g in glob if g[0] < spec.LNF_W] + other + [g for g in glob if g[0] >= spec.LNF_W]
        return out
    monkeypatch.setattr(spec, "stage_tensors", reversed_stages)
    with pytest.raises(AssertionError):
        test_even_stage_default_places_the_hand_listed_layers()
    monkeypatch.setattr(spec, "stage_tensors", real_tensors)
    test_even_stage_default_places_the_hand_listed_layers()


TIED = Model(n_layers=2, hidden=8, n_heads=2, ffn=16, vocab_true=12, max_pos=3, state_elem_bytes=(4, 2), tied_head=True)
TIED_MIX = ((4, "u11"), (2, "index"))


def _tied_golden():
    rows = []
    with open(os.path.join(GOLDEN, "tied_head_p2.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append([(x.rsplit("@", 1)[0], int(x.rsplit("@", 1)[1])) for x in line.split()])
    return rows


def test_tied_head_copy_sits_on_the_last_stage():
    """With a tied output layer and P > 1 the last stage stores the word embeddings too, after the final LayerNorm,
    cut over the tensor-parallel ranks exactly like stage 0's; with P = 1 there is one copy (hand-written lists)."""
    stage0, stage1, single = _tied_golden()
    names = [n for n, _ in spec.NAMES]
    for T in (1, 2):
        par = Parallel(T, 2, 1)
        for t in range(T):
            for p, want in ((0, stage0), (1, stage1)):
                entries, _ = spec.rank_manifest(TIED, par, spec.rank_of(par, t, p, 0))
                for kind in range(2):
                    got = [(names[e.name], e.layer) for e in entries if e.kind == kind]
                    assert got == want, (T, t, p, kind)
            first = [e for e in spec.rank_manifest(TIED, par, spec.rank_of(par, t, 0, 0))[0] if e.name == spec.WORD_EMB]
            last = [e for e in spec.rank_manifest(TIED, par, spec.rank_of(par, t, 1, 0))[0] if e.name == spec.WORD_EMB]
            assert [(e.tensor_id, e.kind, e.full_shape, e.lo, e.hi, e.perm) for e in first] == \
                   [(e.tensor_id, e.kind, e.full_shape, e.lo, e.hi, e.perm) for e in last]
            assert first[0].lo[0] == t * 12 // T and first[0].hi[0] == (t + 1) * 12 // T
    entries, _ = spec.rank_manifest(TIED, Parallel(1, 1, 1), 0)
    assert [(names[e.name], e.layer) for e in entries if e.kind == 0] == single
    # a model without the flag has no second copy
    plain = Model(**{**TIED.__dict__, "tied_head": False})
    assert [e.name for e in spec.rank_manifest(plain, Parallel(1, 2, 1), 1)[0]].count(spec.WORD_EMB) == 0


def test_tied_head_copy_is_a_replica_and_is_dropped_or_made_by_a_reshard():
    """The copy on the last stage holds the same bytes as stage 0's shard; reassembly accepts it as a replica and
    rejects it when it differs; P = 2 -> 1 leaves one copy, P = 1 -> 2 writes the second copy with stage 0's bytes;
    either way every tensor equals the value function at its place."""
    a, b = Parallel(2, 2, 1), Parallel(1, 1, 1)
    src = H.np_bufs(H.make_src_bufs(TIED, a, 13, TIED_MIX))
    for t in range(2):
        r0, r1 = spec.rank_of(a, t, 0, 0), spec.rank_of(a, t, 1, 0)
        for kind in range(2):
            e0 = [e for e in spec.rank_manifest(TIED, a, r0)[0] if e.name == spec.WORD_EMB and e.kind == kind][0]
            e1 = [e for e in spec.rank_manifest(TIED, a, r1)[0] if e.name == spec.WORD_EMB and e.kind == kind][0]
            n = 6 * 8 * e0.elem_bytes
            assert np.array_equal(src[r0][e0.offset:e0.offset + n], src[r1][e1.offset:e1.offset + n])
    one = oreshard.reshard(TIED, a, b, src)
    want = H.np_bufs(H.closed_form_dst_bufs(TIED, a, b, 13, TIED_MIX))
    assert np.array_equal(one[0], want[0])
    back = oreshard.reshard(TIED, b, a, one)                 # P = 1 -> 2: the second copy is made
    assert all(np.array_equal(x, y) for x, y in zip(back, H.np_bufs(H.closed_form_dst_bufs(TIED, b, a, 13, TIED_MIX))))
    for x, y in zip(back, src):                              # and the round trip gives back every tensor byte
        keep = y != H.SRC_GAP
        assert np.array_equal(x[keep], y[keep])
    # a copy that differs from stage 0's is not a replica
    bad = [x.copy() for x in src]
    r1 = spec.rank_of(a, 1, 1, 0)
    e1 = [e for e in spec.rank_manifest(TIED, a, r1)[0] if e.name == spec.WORD_EMB and e.kind == 0][0]
    bad[r1][e1.offset + 5] ^= 0x10
    with pytest.raises(AssertionError):
        oreshard.reshard(TIED, a, b, bad)


def test_pins_catch_a_missing_or_misplaced_tied_copy(monkeypatch):
    real = spec.stage_tensors

    def no_copy(model, par, p):
        return [x for i, x in enumerate(real(model, par, p)) if not (x[0] == spec.WORD_EMB and i > 0)]
    monkeypatch.setattr(spec, "stage_tensors", no_copy)
    with pytest.raises(AssertionError):
        test_tied_head_copy_sits_on_the_last_stage()

    def copy_everywhere(model, par, p):               # also on stages that are not the last, and when P == 1
        out = real(model, par, p)
        if model.tied_head and not (p == par.P - 1 and par.P > 1):
            out = out + [(spec.WORD_EMB, -1)] if p > 0 or par.P == 1 else out
        return out
    monkeypatch.setattr(spec, "stage_tensors", copy_everywhere)
    with pytest.raises(AssertionError):
        test_tied_head_copy_sits_on_the_last_stage()
    monkeypatch.setattr(spec, "stage_tensors", real)
    test_tied_head_copy_sits_on_the_last_stage()
