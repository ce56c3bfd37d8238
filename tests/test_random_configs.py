"""Seeded random small configurations: the planner (its boxes and its tiles interpreted on the CPU) must agree
with the oracle for arbitrary legal (model, source, destination) triples and for arbitrary box partitions of
arbitrary tensors."""
import random

import numpy as np
import pytest
import torch

import paper_2312_05181_amd as tpx
import synth
from oracle import reshard as oreshard
from oracle.spec import Model, Parallel
from tests import helpers as H
from tests import host_exec
from tests.test_generic_ptc import pack, plan_of
from tests.test_planner import plan_for


def _divisors(n):
    return [d for d in range(1, n + 1) if n % d == 0]


def random_case(rng):
    heads = rng.choice([2, 4, 6, 8, 12])
    dh = rng.choice([1, 2, 4, 8])
    h = heads * dh
    ffn = heads * rng.choice([1, 2, 4]) * rng.choice([1, 3])
    layers = rng.choice([1, 2, 3, 4, 6])
    kinds = rng.choice([(4,), (2, 4), (4, 4, 4), (2, 4, 4, 4), (1, 8)])
    div = rng.choice([0, 0, 4, 8])
    vocab = rng.choice([heads * 6, heads * 12]) if div == 0 else rng.randrange(17, 97)
    model = Model(layers, h, heads, ffn, vocab, max_pos=rng.choice([1, 3, 8]), vocab_divisor=div,
                  state_elem_bytes=kinds, tied_head=rng.random() < 0.3)

    def par():
        ts = [t for t in _divisors(heads) if ffn % t == 0 and (div or vocab % t == 0) and t <= 6]
        T = rng.choice(ts)
        P = rng.choice([p for p in (1, 2, 3, 4) if p <= layers])
        D = rng.choice([1, 1, 2, 3])
        if rng.random() < 0.5 or layers % P:
            cuts = sorted(rng.sample(range(0, layers + 1), P - 1)) if P > 1 else []
            stages = tuple([0] + cuts + [layers])
        else:
            stages = None
        shard = rng.randrange(1 << len(kinds)) if D > 1 and rng.random() < 0.5 else 0    # kinds cut over the replicas
        lmap = tuple(rng.randrange(P) for _ in range(layers)) if rng.random() < 0.25 else None      # any layer -> stage map
        return Parallel(T, P, D, stages if lmap is None else None, qkv_layout=rng.choice([0, 0, 1]),
                        w_transposed=rng.choice([0, 0, 0, 1]), shard_kinds=shard, layer_stage=lmap)
    return model, par(), par()


@pytest.mark.parametrize("seed", range(40))
def test_random_gpt_configurations(seed):
    rng = random.Random(1000 + seed)
    model, src, dst = random_case(rng)
    mix = tuple((eb, "index") for eb in model.state_elem_bytes)
    src_bufs = H.np_bufs(H.make_src_bufs(model, src, seed, mix))
    want = oreshard.reshard(model, src, dst, src_bufs)
    plan = plan_for(model, src, dst, opts=dict(tile_bytes=4096))
    for how in (host_exec.run_boxes, host_exec.run_tiles):
        got = [np.full(plan.buffer_bytes(1, r), H.POISON, dtype=np.uint8) for r in range(dst.n_ranks)]
        cover = [np.zeros(len(g), dtype=np.int32) for g in got]
        how(plan, src_bufs, got, cover)
        for r in range(dst.n_ranks):
            assert np.array_equal(got[r], want[r]), (seed, r, model, src, dst)
            assert cover[r].max(initial=0) <= 1
    s = plan.stats()
    assert s["bytes_written"] == oreshard.state_bytes(model, dst)


def random_partition(rng, shape, max_parts):
    """Cut a box into disjoint sub-boxes by recursive bisection along random axes."""
    boxes = [(tuple(0 for _ in shape), tuple(shape))]
    for _ in range(rng.randrange(0, max_parts)):
        i = rng.randrange(len(boxes))
        lo, hi = boxes[i]
        ax = rng.randrange(len(shape))
        if hi[ax] - lo[ax] < 2:
            continue
        cut = rng.randrange(lo[ax] + 1, hi[ax])
        boxes[i] = (lo, hi[:ax] + (cut,) + hi[ax + 1:])
        boxes.append((lo[:ax] + (cut,) + lo[ax + 1:], hi))
    return boxes


def random_collection(rng, tensors, n_ranks):
    ranks = [[] for _ in range(n_ranks)]
    for tid, (shape, kinds, perm) in enumerate(tensors):
        parts = random_partition(rng, shape, 5)
        for lo, hi in parts:
            owners = rng.sample(range(n_ranks), rng.choice([1, 1, 2]) if n_ranks > 1 else 1)   # some boxes are replicated
            for r in owners:
                for k, eb in enumerate(kinds):
                    ranks[r].append((tid, k, eb, shape, lo, hi, perm))
    for per in ranks:
        rng.shuffle(per)
    return pack(ranks)


def random_explicit_case(seed, dims):
    """Random tensors, each cut into random boxes, spread (some replicated) over random ranks, in random
    storage orders on both sides; returns (src manifests, dst manifests, src buffers, oracle result)."""
    rng = random.Random(5000 + seed)
    tensors = []
    for _ in range(rng.randrange(1, 5)):
        nd = rng.randrange(1, 5)
        shape = tuple(rng.choice(dims) for _ in range(nd))
        kinds = rng.choice([(4,), (2, 4), (8,), (1, 2)])
        perm_src = tuple(rng.sample(range(nd), nd))
        tensors.append((shape, kinds, perm_src))
    src = random_collection(rng, tensors, rng.randrange(1, 5))
    tensors_dst = [(s, k, tuple(rng.sample(range(len(s)), len(s)))) for s, k, _ in tensors]   # any storage order
    dst = random_collection(rng, tensors_dst, rng.randrange(1, 6))

    def fill(man, fill_byte):
        out = []
        for entries, n in man:
            b = torch.full((n,), fill_byte, dtype=torch.uint8)
            for e in entries:
                d = H.desc_of(e)
                synth.fill_buffer(b, [d], seed, tuple((d.elem_bytes, "index") for _ in range(d.kind + 1)))
            out.append(b.numpy())
        return out
    a = fill(src, H.SRC_GAP)
    want = oreshard.reshard_ptc(src, dst, a)
    assert all(np.array_equal(x, y) for x, y in zip(want, fill(dst, H.POISON)))      # oracle vs value function
    return src, dst, a, want


@pytest.mark.parametrize("seed", range(40))
def test_random_explicit_collections(seed):
    src, dst, a, want = random_explicit_case(seed, [1, 2, 3, 5, 8, 16, 24])
    plan = plan_of(src, dst, opts=dict(tile_bytes=4096))
    for how in (host_exec.run_boxes, host_exec.run_tiles):
        got = [np.full(n, H.POISON, dtype=np.uint8) for _, n in dst]
        how(plan, a, got)
        for r in range(len(dst)):
            assert np.array_equal(got[r], want[r]), (seed, r)


@pytest.mark.gpu
@pytest.mark.parametrize("dims", [[1, 2, 3, 5, 8, 16, 24], [1, 3, 8, 24, 64, 136, 200]], ids=["small", "large"])
@pytest.mark.parametrize("seed", range(40))
def test_random_explicit_collections_gpu(cuda, seed, dims):
    """The same random collections through the kernel: gathers, ragged and full transposing sub-tiles,
    1- to 16-byte units."""
    from tests import gpu_util as G
    src, dst, a, want = random_explicit_case(seed, dims)
    print("seed", seed, "dims", dims[-1], "bytes", sum(n for _, n in dst), flush=True)
    plan = plan_of(src, dst, opts=dict(tile_bytes=4096 if dims[-1] < 100 else 131072))
    got, _ = G.execute(plan, [torch.from_numpy(x).cuda() for x in a])
    torch.cuda.synchronize()
    for r in range(len(dst)):
        assert np.array_equal(got[r].cpu().numpy(), want[r]), (seed, r)


@pytest.mark.gpu
@pytest.mark.parametrize("seed", range(40))
def test_random_gpt_configurations_gpu(cuda, seed):
    from tests import gpu_util as G
    rng = random.Random(1000 + seed)
    model, src, dst = random_case(rng)
    print("seed", seed, model, src, dst, flush=True)
    mix = tuple((eb, "index") for eb in model.state_elem_bytes)
    src_cpu = H.make_src_bufs(model, src, seed, mix)
    want = oreshard.reshard(model, src, dst, H.np_bufs(src_cpu))
    plan = plan_for(model, src, dst, opts=dict(tile_bytes=4096))
    got, _ = G.execute(plan, [b.cuda() for b in src_cpu])
    torch.cuda.synchronize()
    for r in range(dst.n_ranks):
        assert np.array_equal(got[r].cpu().numpy(), want[r]), (seed, r)


@pytest.mark.gpu
def test_largest_rank_count(cuda):
    """128 buffers per side (the limit of the kernel's pointer table): T 8 x P 4 x D 4 -> T 4 x P 8 x D 4."""
    from tests import gpu_util as G
    model = Model(n_layers=8, hidden=64, n_heads=8, ffn=128, vocab_true=64, max_pos=4, state_elem_bytes=(2, 4))
    src, dst = Parallel(8, 4, 4), Parallel(4, 8, 4)
    assert src.n_ranks == dst.n_ranks == 128
    mix = ((2, "index"), (4, "u11"))
    src_cpu = H.make_src_bufs(model, src, 2, mix)
    want = oreshard.reshard(model, src, dst, H.np_bufs(src_cpu))
    plan = plan_for(model, src, dst)
    got, _ = G.execute(plan, [b.cuda() for b in src_cpu])
    torch.cuda.synchronize()
    for r in range(dst.n_ranks):
        assert np.array_equal(got[r].cpu().numpy(), want[r]), r
    with pytest.raises(tpx.TpxError):
        plan_for(model, Parallel(8, 4, 8), dst)
