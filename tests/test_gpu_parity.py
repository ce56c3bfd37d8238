"""Parity of the HIP path (through the C ABI) with the CPU oracle, bit for bit.

Small cases: every destination byte is compared with the oracle's output (including the poison in
alignment gaps).  Full-size workloads: every destination tensor is compared on the GPU with its
closed-form contents (the value function evaluated at the oracle's layout), gaps are checked to be
untouched, and a sample of tensors goes through the CPU oracle itself."""
import numpy as np
import pytest
import torch

import paper_2312_05181_amd as tpx
import synth
from oracle import dataset as ods
from oracle import reshard as oreshard
from oracle import spec
from oracle.spec import Model, Parallel
from tests import gpu_util as G
from tests import helpers as H
from tests.test_planner import ODD, ODD_MIX, PAIRS, SMALL, SMALL_MIX, WIDE, plan_for

pytestmark = pytest.mark.gpu


def _check_small(model, mix, src, dst, seed=17, **plan_kw):
    src_cpu = H.make_src_bufs(model, src, seed, mix)
    want = oreshard.reshard(model, src, dst, H.np_bufs(src_cpu))
    plan = plan_for(model, src, dst, **plan_kw)
    src_gpu = [b.cuda() for b in src_cpu]
    got, _ = G.execute(plan, src_gpu)
    torch.cuda.synchronize()
    for r, (g, w) in enumerate(zip(got, want)):
        assert np.array_equal(g.cpu().numpy(), w), f"rank {r}"
    for a, b in zip(src_gpu, src_cpu):          # sources are only read
        assert torch.equal(a.cpu(), b)
    return plan


@pytest.mark.parametrize("model,mix,src,dst", PAIRS)
def test_small_reshards_match_oracle(cuda, model, mix, src, dst):
    """Odd sizes: exercises 2-, 4-, 8- and 16-byte units, fills, transposes and gathers."""
    print("case", model.hidden, src, dst, flush=True)
    _check_small(model, mix, src, dst)


@pytest.mark.parametrize("tile_bytes", [4096, 65536])
@pytest.mark.parametrize("src,dst", [(Parallel(2, 2, 1), Parallel(4, 1, 2)), (Parallel(8, 1, 1), Parallel(1, 2, 1)),
                                     (Parallel(4, 1, 1), Parallel(8, 2, 1, qkv_layout=1)),
                                     (Parallel(2, 1, 1, w_transposed=1), Parallel(4, 2, 1))])
def test_several_tiles_and_ragged_tails(cuda, tile_bytes, src, dst):
    """16-byte path with many tiles per box, 2-D tiles with a ragged last tile, tied embedding copy."""
    print("case", tile_bytes, src, dst, flush=True)
    plan = _check_small(WIDE, synth.MIX_GPT, src, dst, opts=dict(tile_bytes=tile_bytes))
    assert plan.num_tiles() > 100


@pytest.mark.parametrize("variant", [u | (n * 24) | (t << 5) for t in range(3) for n in range(2) for u in (2, 3, 4)])
def test_every_kernel_variant(cuda, variant):
    print("variant", variant, flush=True)
    tpx.tpx_set_option("variant", variant)
    try:
        _check_small(WIDE, synth.MIX_GPT, Parallel(4, 1, 1), Parallel(2, 2, 1), opts=dict(tile_bytes=16384))
        _check_small(ODD, ODD_MIX, Parallel(3, 1, 1), Parallel(4, 1, 1), opts=dict(tile_bytes=16384))
    finally:
        tpx.tpx_set_option("variant", 0)


def test_tiny_config_and_layout_change(cuda):
    """Workload 1 (Tiny GPT, (2,1,1) -> (4,2,1)) and the same with a qkv-major destination."""
    model, src, dst, mix, seed = H.CONFIGS[1]
    _check_small(model, mix, src, dst, seed)
    _check_small(model, mix, src, Parallel(4, 2, 1, qkv_layout=1), seed)
    _check_small(model, mix, Parallel(2, 1, 1, qkv_layout=1), Parallel(4, 2, 1, w_transposed=1), seed)


def test_plan_can_be_executed_repeatedly_and_round_trips(cuda):
    model, mix = WIDE, synth.MIX_GPT
    a, b = Parallel(2, 2, 1), Parallel(4, 1, 2)
    src = [x.cuda() for x in H.make_src_bufs(model, a, 9, mix)]
    fwd, back = plan_for(model, a, b), plan_for(model, b, a)
    mid, ws = G.execute(fwd, src)
    mid2, _ = G.execute(fwd, src, workspace=ws)               # same workspace, second launch
    torch.cuda.synchronize()
    assert all(torch.equal(x, y) for x, y in zip(mid, mid2))
    out, _ = G.execute(back, mid)
    torch.cuda.synchronize()
    for r in range(a.n_ranks):                                # A -> B -> A is the identity on tensor bytes
        for e in spec.rank_manifest(model, a, r)[0]:
            d = H.desc_of(e)
            assert torch.equal(out[r][d.offset:d.offset + d.nbytes], src[r][d.offset:d.offset + d.nbytes])


def test_failure_recovery_reads_only_survivors(cuda):
    model, mix = SMALL, SMALL_MIX
    src, dst = Parallel(2, 2, 2), Parallel(2, 1, 1)
    alive = [1] * src.n_ranks
    for t in range(2):
        alive[spec.rank_of(src, t, 0, 0)] = 0
        alive[spec.rank_of(src, t, 1, 1)] = 0
    src_cpu = H.make_src_bufs(model, src, 5, mix)
    want = oreshard.reshard(model, src, dst, H.np_bufs(src_cpu))
    plan = plan_for(model, src, dst, rank_alive=alive)
    src_gpu = [b.cuda() if alive[r] else torch.empty(0, dtype=torch.uint8, device="cuda") for r, b in enumerate(src_cpu)]
    got, _ = G.execute(plan, src_gpu)            # lost ranks are passed as NULL pointers
    torch.cuda.synchronize()
    assert all(np.array_equal(g.cpu().numpy(), w) for g, w in zip(got, want))


def test_rebuild_only_the_lost_ranks(cuda):
    """(4,2,2) with one replica of every share lost: only those eight ranks are rebuilt; the survivors' destination
    pointers are NULL and nothing is written for them."""
    model, mix = SMALL, SMALL_MIX
    cfg = Parallel(4, 2, 2)
    gone = {spec.rank_of(cfg, t, p, (t + p) % 2) for t in range(4) for p in range(2)}
    alive = [0 if r in gone else 1 for r in range(16)]
    need = [1 - a for a in alive]
    src_cpu = H.make_src_bufs(model, cfg, 5, mix)
    want = oreshard.reshard(model, cfg, cfg, H.np_bufs(src_cpu))
    plan = plan_for(model, cfg, cfg, dst_alive=need, rank_alive=alive)
    empty = torch.empty(0, dtype=torch.uint8, device="cuda")
    src_gpu = [b.cuda() if alive[r] else empty for r, b in enumerate(src_cpu)]
    dst_gpu = [G.alloc(plan.buffer_bytes(1, r), H.POISON) if need[r] else empty for r in range(16)]
    G.execute(plan, src_gpu, dst_bufs=dst_gpu)
    torch.cuda.synchronize()
    for r in range(16):
        if need[r]:
            assert np.array_equal(dst_gpu[r].cpu().numpy(), want[r]), r
    with pytest.raises(tpx.TpxError):        # a rank that is to be built needs its buffer
        bad = list(dst_gpu)
        bad[min(gone)] = empty
        G.execute(plan, src_gpu, dst_bufs=bad)
    torch.cuda.synchronize()


@pytest.mark.parametrize("shift", [16, 48, 240])
def test_rank_buffers_aligned_to_16_bytes_only(cuda, shift):
    """The contract asks for 16-byte aligned rank buffers, not more: every buffer starts `shift` bytes into
    its allocation (merge, multicast, fill and transposing tiles included)."""
    for model, mix, a, b in ((WIDE, synth.MIX_GPT, Parallel(2, 2, 1), Parallel(4, 1, 2)),
                             (ODD, ODD_MIX, Parallel(3, 1, 1), Parallel(4, 2, 1, w_transposed=1))):
        src_cpu = H.make_src_bufs(model, a, 29, mix)
        want = oreshard.reshard(model, a, b, H.np_bufs(src_cpu))
        plan = plan_for(model, a, b)
        src_gpu = []
        for x in src_cpu:
            t = G.alloc(x.numel() + 256, 0)
            t[shift:shift + x.numel()] = x.cuda()
            src_gpu.append(t[shift:shift + x.numel()])
        dst_gpu = [G.alloc(plan.buffer_bytes(1, r) + 256, H.POISON)[shift:shift + plan.buffer_bytes(1, r)] for r in range(b.n_ranks)]
        assert all(t.data_ptr() % 256 == shift for t in src_gpu + dst_gpu)
        G.execute(plan, src_gpu, dst_bufs=dst_gpu)
        torch.cuda.synchronize()
        for r in range(b.n_ranks):
            assert np.array_equal(dst_gpu[r].cpu().numpy(), want[r]), (shift, r)


def test_execute_argument_errors(cuda):
    plan = plan_for(SMALL, Parallel(2, 1, 1), Parallel(1, 1, 1))
    src = [G.alloc(plan.buffer_bytes(0, r), 0) for r in range(2)]
    dst = [G.alloc(plan.buffer_bytes(1, 0), 0)]
    ws = G.alloc(plan.workspace_bytes() + 64)
    E = tpx.binding

    def status(fn):
        with pytest.raises(tpx.TpxError) as err:
            fn()
        return err.value.status
    assert status(lambda: tpx.tpx_execute(plan, [src[0].data_ptr(), 0], [dst[0].data_ptr()], ws.data_ptr())) == E.TPX_ERR_INVALID_ARG
    assert status(lambda: tpx.tpx_execute(plan, [src[0].data_ptr() + 4, src[1].data_ptr()], [dst[0].data_ptr()], ws.data_ptr())) == E.TPX_ERR_MISALIGNED
    assert status(lambda: tpx.tpx_execute(plan, [s.data_ptr() for s in src], [dst[0].data_ptr() + 8], ws.data_ptr())) == E.TPX_ERR_MISALIGNED
    assert status(lambda: tpx.tpx_execute(plan, [s.data_ptr() for s in src], [dst[0].data_ptr()], ws.data_ptr() + 8)) == E.TPX_ERR_MISALIGNED
    assert status(lambda: tpx.tpx_execute(plan, [s.data_ptr() for s in src], [dst[0].data_ptr()], 0)) == E.TPX_ERR_INVALID_ARG
    assert status(lambda: tpx.tpx_probe_copy(dst[0].data_ptr() + 4, src[0].data_ptr(), 16)) == E.TPX_ERR_MISALIGNED
    torch.cuda.synchronize()


def test_two_plans_take_turns_on_one_workspace(cuda):
    """Plans A and B alternate on one workspace (A, B, A, A, B): the library knows whose tables it last copied there
    and copies again when they are the other plan's, so every execute moves its own plan's bytes."""
    model, mix = SMALL, SMALL_MIX
    a, b1, b2 = Parallel(2, 1, 1), Parallel(1, 2, 1), Parallel(2, 2, 1)
    src_cpu = H.make_src_bufs(model, a, 3, mix)
    src = [x.cuda() for x in src_cpu]
    plans = {"A": plan_for(model, a, b1), "B": plan_for(model, a, b2)}
    want = {"A": oreshard.reshard(model, a, b1, H.np_bufs(src_cpu)), "B": oreshard.reshard(model, a, b2, H.np_bufs(src_cpu))}
    ws = G.alloc(max(p.workspace_bytes() for p in plans.values()))
    stream = torch.cuda.current_stream().cuda_stream
    for turn in "ABAAB":
        got, _ = G.execute(plans[turn], src, workspace=ws)
        plans[turn].workspace_check(ws.data_ptr(), stream)
        assert all(np.array_equal(g.cpu().numpy(), w) for g, w in zip(got, want[turn])), turn
    tpx.tpx_workspace_forget(ws.data_ptr())


def test_overwritten_workspace_moves_nothing_and_is_reported(cuda):
    """A workspace that somebody else overwrote since the upload (which the library cannot know): the launch must not
    follow what is there now; tpx_workspace_check reports it, after which the next execute copies the tables again."""
    model, mix = SMALL, SMALL_MIX
    a, b = Parallel(2, 1, 1), Parallel(1, 2, 1)
    src_cpu = H.make_src_bufs(model, a, 3, mix)
    want = oreshard.reshard(model, a, b, H.np_bufs(src_cpu))
    src = [x.cuda() for x in src_cpu]
    first, other = plan_for(model, a, b), plan_for(model, a, Parallel(2, 2, 1))
    ws = G.alloc(max(first.workspace_bytes(), other.workspace_bytes()))
    ws2 = G.alloc(other.workspace_bytes())
    stream = torch.cuda.current_stream().cuda_stream
    got, _ = G.execute(first, src, workspace=ws)
    first.workspace_check(ws.data_ptr(), stream)
    assert all(np.array_equal(g.cpu().numpy(), w) for g, w in zip(got, want))
    other.prepare(ws2.data_ptr(), stream)
    ws[:ws2.numel()].copy_(ws2)                                  # the other plan's tables, behind the library's back
    stale, _ = G.execute(first, src, workspace=ws)               # the library still believes ws holds `first`
    torch.cuda.synchronize()
    assert all(bool((x == H.POISON).all()) for x in stale)       # nothing was written
    with pytest.raises(tpx.TpxError) as err:
        first.workspace_check(ws.data_ptr(), stream)
    assert err.value.status == tpx.binding.TPX_ERR_STALE_WORKSPACE
    got, _ = G.execute(first, src, workspace=ws)                 # the check made the library forget: uploaded again
    first.workspace_check(ws.data_ptr(), stream)
    assert all(np.array_equal(g.cpu().numpy(), w) for g, w in zip(got, want))
    ws.zero_()                                                   # garbage instead of any plan
    stale, _ = G.execute(first, src, workspace=ws)
    torch.cuda.synchronize()
    assert all(bool((x == H.POISON).all()) for x in stale)
    tpx.tpx_workspace_forget(ws.data_ptr())                      # told so, it uploads again
    got, _ = G.execute(first, src, workspace=ws)
    first.workspace_check(ws.data_ptr(), stream)
    assert all(np.array_equal(g.cpu().numpy(), w) for g, w in zip(got, want))
    tpx.tpx_workspace_forget(ws.data_ptr())
    tpx.tpx_workspace_forget(ws2.data_ptr())


def test_one_plan_executed_from_several_threads(cuda):
    """tpx_execute takes the plan as const: four host threads launch the same plan on the same prepared workspace,
    each into its own destination buffers, on the same stream."""
    import threading
    model, mix = WIDE, synth.MIX_GPT
    a, b = Parallel(2, 2, 1), Parallel(4, 1, 2)
    src_cpu = H.make_src_bufs(model, a, 9, mix)
    want = oreshard.reshard(model, a, b, H.np_bufs(src_cpu))
    src = [x.cuda() for x in src_cpu]
    plan = plan_for(model, a, b)
    ws = G.alloc(plan.workspace_bytes())
    stream = torch.cuda.current_stream().cuda_stream
    outs = [[G.alloc(plan.buffer_bytes(1, r), H.POISON) for r in range(b.n_ranks)] for _ in range(4)]
    torch.cuda.synchronize()
    errors = []

    def run(i):
        try:
            for _ in range(3):
                tpx.tpx_execute(plan, [x.data_ptr() for x in src], [x.data_ptr() for x in outs[i]], ws.data_ptr(), stream)
        except Exception as e:      # noqa: BLE001
            errors.append(e)
    threads = [threading.Thread(target=run, args=(i,)) for i in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors
    for got in outs:
        assert all(np.array_equal(g.cpu().numpy(), w) for g, w in zip(got, want))
    tpx.tpx_workspace_forget(ws.data_ptr())


def test_probe_copy(cuda):
    for n in (16, 4096 + 48, 1 << 24):
        a = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda")
        b = torch.zeros(n + 16, dtype=torch.uint8, device="cuda")
        tpx.tpx_probe_copy(b.data_ptr(), a.data_ptr(), n, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert torch.equal(a, b[:n]) and not b[n:].any()


# ---------------------------------------------------------------------------------------------
# the full-size workloads, in the launch configuration the benchmark times
# ---------------------------------------------------------------------------------------------
def test_read_and_fill_probes(cuda):
    """The write-only yardstick writes exactly the bytes it is given, the read-only one touches nothing but (at most) its
    16-byte sink; both refuse what they cannot take."""
    n = (1 << 20) + 48                                   # a ragged last workgroup
    buf = G.alloc(n + 64, 0x11)
    stream = torch.cuda.current_stream().cuda_stream
    tpx.tpx_probe_fill(buf.data_ptr() + 16, n, 0xC3C3C3C3, stream)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert (host[:16] == 0x11).all() and (host[16:16 + n] == 0xC3).all() and (host[16 + n:] == 0x11).all()
    sink = G.alloc(16, 0)
    tpx.tpx_probe_read(buf.data_ptr() + 16, n, sink.data_ptr(), stream)
    torch.cuda.synchronize()
    assert np.array_equal(buf.cpu().numpy(), host)
    tpx.tpx_probe_read(buf.data_ptr(), 0, sink.data_ptr(), stream)
    for bad in (lambda: tpx.tpx_probe_fill(buf.data_ptr() + 8, 64, 0, stream), lambda: tpx.tpx_probe_read(buf.data_ptr(), 24, sink.data_ptr(), stream),
                lambda: tpx.tpx_probe_read(buf.data_ptr(), 64, 0, stream), lambda: tpx.tpx_probe_fill(0, 64, 0, stream)):
        with pytest.raises(tpx.TpxError):
            bad()


def _sample_ids(model):
    L = model.n_layers
    ids = [0, 1, 2, 3]
    for layer in sorted({0, L // 2 - 1, L - 1}):
        ids += [4 + layer * 12 + k for k in range(12)]
    return ids


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_full_size_workload(cuda, cfg):
    model, src, dst, mix, seed = H.CONFIGS[cfg]
    print("workload", cfg, "allocating", flush=True)
    plan = plan_for(model, src, dst)
    src_descs = H.manifest_descs(model, src)
    src_gpu = []
    for r, (descs, n) in enumerate(src_descs):
        assert plan.buffer_bytes(0, r) == n
        b = G.alloc(n, H.SRC_GAP)
        synth.fill_buffer(b, descs, seed, mix)
        src_gpu.append(b)
    print("workload", cfg, "executing", plan.stats(), flush=True)
    got, _ = G.execute(plan, src_gpu)
    torch.cuda.synchronize()
    print("workload", cfg, "checking closed form", flush=True)
    assert H.closed_form_mismatches(got, model, src, dst, seed, mix) == 0
    for b, (descs, n) in zip(got, H.manifest_descs(model, dst)):
        assert H.gaps_untouched(b, descs, H.POISON)
    # a sample of tensors through the CPU oracle itself
    print("workload", cfg, "checking sampled tensors against the oracle", flush=True)
    src_lay, dst_lay = oreshard.Layout(model, src), oreshard.Layout(model, dst)

    def read(rank, off, n):
        return src_gpu[rank][off:off + n].cpu().numpy()

    for tid in _sample_ids(model):
        for kind in range(len(model.state_elem_bytes)):
            for rank, e, block in oreshard.reshard_tensor(model, src, dst, src_lay, dst_lay, tid, kind, read):
                have = got[rank][e.offset:e.offset + block.nbytes].cpu().numpy()
                assert np.array_equal(have, block.reshape(-1).view(np.uint8)), (tid, kind, rank)
    del got, src_gpu
    torch.cuda.empty_cache()


@pytest.mark.parametrize("cfg,tile_bytes,variant", [(2, 1 << 18, 0), (2, 1 << 22, 0), (5, 1 << 20, 0), (2, 1 << 20, 26)])
def test_full_size_with_tiles_of_several_passes(cuda, cfg, tile_bytes, variant):
    """Tiles larger than what a workgroup holds in flight (256 KiB to 2 MiB against 128 KiB at most; with the smallest
    kernel shape, 256 threads x 4 loads, 64 passes per tile), on jobs large enough that the planner keeps them: copies,
    equal merges (workload 2) and merges of unequal column blocks with fills (workload 5)."""
    model, src, dst, _, seed = H.CONFIGS[cfg]
    plan = plan_for(model, src, dst, opts=dict(tile_bytes=tile_bytes))
    biggest = max(t.nrows * (t.run_units << t.unit_log2) for t in plan.tiles()[::97])
    assert biggest > (1 << 17) and biggest <= tile_bytes
    tpx.tpx_set_option("variant", variant)
    try:
        _run_full_size(f"workload {cfg}, tiles of up to {tile_bytes} bytes, variant {variant}", model, src, dst, seed, plan)
    finally:
        tpx.tpx_set_option("variant", 0)


@pytest.mark.parametrize("cfg", [2, 5])
def test_full_size_round_trip_and_composition(cuda, cfg):
    """Properties that hold at any size, in the launch configuration the benchmark times: A -> B -> A gives
    back every tensor byte of A, and A -> B -> C lands the same bytes as A -> C (workload 5 grows the padded
    vocabulary on the way out: the way back drops the zero rows again, and C, padded like B, gets the same
    zero rows either way)."""
    model, a, b, mix, seed = H.CONFIGS[cfg]
    c = Parallel(1, 2, 1) if cfg == 2 else Parallel(6, 1, 1)
    src_descs = H.manifest_descs(model, a)
    src_gpu = []
    for descs, n in src_descs:
        buf = G.alloc(n, H.SRC_GAP)
        synth.fill_buffer(buf, descs, seed, mix)
        src_gpu.append(buf)
    print("workload", cfg, "A->B", flush=True)
    mid, _ = G.execute(plan_for(model, a, b), src_gpu)
    print("workload", cfg, "B->A", flush=True)
    back, _ = G.execute(plan_for(model, b, a), mid)
    torch.cuda.synchronize()
    for r, (descs, n) in enumerate(src_descs):
        for d in descs:
            assert torch.equal(back[r][d.offset:d.offset + d.nbytes], src_gpu[r][d.offset:d.offset + d.nbytes]), (r, d.tensor_id, d.kind)
    del back
    torch.cuda.empty_cache()
    print("workload", cfg, "B->C and A->C", flush=True)
    via, _ = G.execute(plan_for(model, b, c), mid)
    direct, _ = G.execute(plan_for(model, a, c), src_gpu)
    torch.cuda.synchronize()
    for r in range(c.n_ranks):        # whole buffers: tensor bytes and the untouched poison in the gaps
        assert torch.equal(via[r], direct[r]), r
    assert H.closed_form_mismatches(direct, model, a, c, seed, mix) == 0
    del via, direct, mid, src_gpu
    torch.cuda.empty_cache()


# ---------------------------------------------------------------------------------------------
# dataset state
# ---------------------------------------------------------------------------------------------
def _dataset_case(n, Bsz, D, D2, s, seed=6, eb=8):
    Gord = synth.epoch_order(n, seed) if n else np.zeros(0, dtype=np.uint64)
    if eb == 16:       # (offset, length) entries (paper section 5.2): two 64-bit words per sample, rows of the index
        Gord = np.stack([Gord * np.uint64(4096), Gord % np.uint64(1000) + np.uint64(1)], axis=1)
    parts = ods.partition(Gord, Bsz, D)
    cur = ods.cursors_after(n, Bsz, D, s)
    want_parts, want_cur = ods.repartition(parts, cur, Bsz, D2)
    plan = tpx.tpx_plan_dataset(n, Bsz, D, D2, cur, index_elem_bytes=eb)
    assert plan.dst_cursors == want_cur
    empty = torch.empty(0, dtype=torch.uint8, device="cuda")
    src = [torch.from_numpy(np.ascontiguousarray(p).reshape(-1).view(np.uint8)).cuda() if p.size else empty for p in parts]
    assert [plan.buffer_bytes(0, j) for j in range(D)] == [x.numel() for x in src]
    got, _ = G.execute(plan, src)
    torch.cuda.synchronize()
    for j in range(D2):
        assert np.array_equal(got[j].cpu().numpy().view(np.uint64), np.ascontiguousarray(want_parts[j]).reshape(-1)), j


@pytest.mark.parametrize("n,Bsz,D,D2,s", [(100, 24, 6, 4, 2), (101, 24, 4, 6, 3), (7, 12, 6, 4, 1), (0, 12, 2, 3, 0),
                                          (768 * 50 + 256, 768, 6, 4, 20), (100000, 768, 4, 6, 130), (1000, 48, 6, 6, 7)])
def test_dataset_small(cuda, n, Bsz, D, D2, s):
    print("dataset", n, Bsz, D, D2, s, flush=True)
    _dataset_case(n, Bsz, D, D2, s)


def test_dataset_random(cuda):
    """300 seeded random repartitionings: 1 to 12 replicas on either side, any global batch both divide, any step of the epoch
    (also none consumed, all consumed, fewer samples than one batch, no samples), 8- and 16-byte entries."""
    import math
    import random
    rng = random.Random(77)
    for i in range(300):
        D, D2 = rng.randrange(1, 13), rng.randrange(1, 13)
        Bsz = math.lcm(D, D2) * rng.randrange(1, 9)
        n = rng.choice([0, rng.randrange(1, Bsz + 1), rng.randrange(1, 40 * Bsz), rng.randrange(1, 3000 * Bsz)])
        s = rng.randrange(0, -(-n // Bsz) + 1)
        eb = rng.choice([8, 16])
        print("dataset", i, (n, Bsz, D, D2, s, eb), flush=True)
        _dataset_case(n, Bsz, D, D2, s, seed=i, eb=eb)


@pytest.mark.parametrize("eb", [8, 16])
def test_dataset_full_size(cuda, eb):
    """10^8 samples, 6 -> 4 replicas after 65,000 steps: ids (8 bytes) and (offset, length) pairs (16 bytes)."""
    c = H.DATASET_CFG
    print("dataset full size", c, "entry bytes", eb, flush=True)
    _dataset_case(c["n_samples"], c["global_batch"], c["D_src"], c["D_dst"], c["steps_done"], c["seed"], eb)


@pytest.mark.parametrize("n,Bsz,D,D2,s", [(100, 24, 6, 4, 2), (7, 12, 6, 4, 1), (768 * 50 + 256, 768, 6, 4, 20), (100000, 768, 4, 6, 130)])
def test_dataset_pairs_small(cuda, n, Bsz, D, D2, s):
    _dataset_case(n, Bsz, D, D2, s, eb=16)


# ---------------------------------------------------------------------------------------------
# the paper's own reconfigurations (sections 6.2, 6.3, 6.6, 6.8) at full size
# ---------------------------------------------------------------------------------------------
def _bench_case(name):
    """(model, src, dst, seed) of a workload of bench.py in the oracle's terms."""
    import bench
    mk_, s_, d_, _, seed = bench.WORKLOADS[name]
    model = Model(mk_["n_layers"], mk_["hidden"], mk_["n_heads"], mk_["ffn"], mk_["vocab_true"], mk_.get("max_pos", 1024),
                  mk_.get("vocab_divisor", 0), tuple(mk_["state_elem_bytes"]))

    def par(c):
        return Parallel(c["T"], c["P"], c["D"], c.get("stage_first_layer"), c.get("qkv_layout", 0), c.get("w_transposed", 0),
                        c.get("shard_kinds", 0), c.get("layer_stage"))
    return model, par(s_), par(d_), seed, s_.get("rank_alive"), d_.get("rank_alive")


def _run_full_size(name, model, src, dst, seed, plan, src_alive=None, dst_built=None):
    """One full-size reshard in the launch configuration the benchmark times, checked three ways: every destination
    tensor against its closed-form contents (on the GPU), the gaps between tensors untouched, and a sample of tensors
    (embeddings, final LayerNorm, three layers, every state kind) through the CPU oracle itself.  Source ranks that
    are lost get no buffer at all; destination ranks that are not built get none either."""
    mix = synth.MIX_GPT
    empty = torch.empty(0, dtype=torch.uint8, device="cuda")
    print(name, "allocating", plan.stats(), flush=True)
    src_gpu = []
    for r, (descs, n) in enumerate(H.manifest_descs(model, src)):
        assert plan.buffer_bytes(0, r) == n
        if src_alive is not None and not src_alive[r]:
            src_gpu.append(empty)
            continue
        b = G.alloc(n, H.SRC_GAP)
        synth.fill_buffer(b, descs, seed, mix)
        src_gpu.append(b)
    dst_descs = H.manifest_descs(model, dst)
    dst_gpu = [G.alloc(n, H.POISON) if dst_built is None or dst_built[r] else empty for r, (_, n) in enumerate(dst_descs)]
    print(name, "executing", flush=True)
    G.execute(plan, src_gpu, dst_bufs=dst_gpu)
    torch.cuda.synchronize()
    print(name, "checking closed form", flush=True)
    zero_rule = H._zero_rule(model, src)
    for r, (descs, n) in enumerate(dst_descs):
        if dst_built is not None and not dst_built[r]:
            continue
        assert synth.count_mismatch(dst_gpu[r], descs, seed, mix, zero_from_row=zero_rule) == 0, r
        assert H.gaps_untouched(dst_gpu[r], descs, H.POISON), r
    print(name, "checking sampled tensors against the oracle", flush=True)
    src_lay, dst_lay = oreshard.Layout(model, src), oreshard.Layout(model, dst)

    def read(rank, off, n):
        if src_alive is not None and not src_alive[rank]:
            # a lost rank: the oracle's "any replica" is a surviving rank with the same (t, p), whose buffer has the same layout
            t, p, _ = spec.coords_of(src, rank)
            rank = next(q for q in (spec.rank_of(src, t, p, d) for d in range(src.D)) if src_alive[q])
        return src_gpu[rank][off:off + n].cpu().numpy()

    for tid in _sample_ids(model):
        for kind in range(len(model.state_elem_bytes)):
            for rank, e, block in oreshard.reshard_tensor(model, src, dst, src_lay, dst_lay, tid, kind, read):
                if dst_built is not None and not dst_built[rank]:
                    continue
                have = dst_gpu[rank][e.offset:e.offset + block.nbytes].cpu().numpy()
                assert np.array_equal(have, block.reshape(-1).view(np.uint8)), (tid, kind, rank)
    del dst_gpu, src_gpu
    torch.cuda.empty_cache()


def _paper_pairs():
    import bench
    return list(bench.PAPER_PAIRS) + list(bench.SHARDED_PAIRS)   # plus the sharded-optimizer-state reshards, checked the same way


@pytest.mark.parametrize("name", _paper_pairs())
def test_paper_reconfiguration_pairs(cuda, name):
    """Data-, pipeline- and tensor-parallel changes, redeployment and the elastic-scaling sequence of the
    paper's evaluation (sections 6.2, 6.3, 6.6, 6.8) at the 1.3B, 2.7B, 6.7B and BERT-large shapes: every destination
    tensor equals its closed-form contents, gaps stay untouched, sampled tensors equal the oracle's, and replicated
    destinations are written from a single read (multicast moves)."""
    model, src, dst, seed, _, _ = _bench_case(name)
    plan = plan_for(model, src, dst)
    st = plan.stats()
    if src.D == 1 and dst.D > 1 and src.T == dst.T and src.P == dst.P:
        assert st["bytes_read"] * dst.D == st["bytes_written"]        # read once, written D' times
    assert st["bytes_read"] <= st["bytes_written"]
    _run_full_size(name, model, src, dst, seed, plan)


def test_single_rank_redeploy_moves_one_whole_buffer(cuda):
    """6.7B shape on one rank, redeployed to one rank (section 6.3's redeployment at T = P = D = 1): the whole 93 GB buffer
    coalesces into a single contiguous move, longer than a 32-bit count of 16-byte units, which the planner cuts into
    several runs of tiles."""
    model, src, dst = H.GPT_6_7B, Parallel(1, 1, 1), Parallel(1, 1, 1)
    plan = plan_for(model, src, dst)
    st = plan.stats()
    assert st["n_boxes"] == 1 and st["bytes_read"] == st["bytes_written"] == 93_161_635_840
    _run_full_size("gpt6.7b_(1,1,1)->(1,1,1)", model, src, dst, 4, plan)


def _layout_pairs():
    import bench
    return list(bench.LAYOUT_PAIRS)


@pytest.mark.parametrize("name", _layout_pairs())
def test_layout_changing_reshards_full_size(cuda, name):
    """1.3B shape with a qkv-major or a transposed ([in, out]) destination: the strided relayout and the LDS-staged
    transposing tiles at the size the benchmark times them."""
    model, src, dst, seed, _, _ = _bench_case(name)
    plan = plan_for(model, src, dst)
    kinds = {b.kind for b in plan.boxes()}
    assert (2 in kinds) == bool(dst.w_transposed)       # TPX_BOX_TRANSPOSE
    _run_full_size(name, model, src, dst, seed, plan)


def test_recovery_full_size(cuda):
    """2.7B shape, (4,2,2) with one replica of every (t, p) share lost (paper sections 5.3 and 6.4): the eight lost ranks are
    rebuilt from their surviving replicas; lost ranks have no source buffer, survivors no destination buffer."""
    import bench
    name = next(iter(bench.RECOVERY))
    model, src, dst, seed, alive, built = _bench_case(name)
    assert sum(alive) == 8 and [1 - a for a in alive] == list(built)
    plan = plan_for(model, src, dst, dst_alive=built, rank_alive=alive)
    assert {b.dst_rank for b in plan.boxes()} == {r for r in range(16) if built[r]}
    assert {b.src_rank for b in plan.boxes()} <= {r for r in range(16) if alive[r]}
    _run_full_size(name, model, src, dst, seed, plan, src_alive=alive, dst_built=built)


def test_shared_reads_full_size(cuda):
    """BERT-large-shape (1,1,4) -> (1,1,8) with share_reads: one 8-way multicast move per piece, every replica
    complete (closed form, sampled tensors through the oracle), gaps untouched, one fifth of the reads of the
    locality plan."""
    name = "bert-large_(1,1,4)->(1,1,8)"
    model, src, dst, seed, _, _ = _bench_case(name)
    local = plan_for(model, src, dst).stats()
    plan = plan_for(model, src, dst, opts=dict(share_reads=1))
    st = plan.stats()
    assert st["bytes_written"] == local["bytes_written"] == 8 * st["bytes_read"] and local["bytes_read"] == 5 * st["bytes_read"]
    _run_full_size(name + " share_reads", model, src, dst, seed, plan)


def test_multicast_small(cuda):
    """Replicated destinations on odd-sized models: copy, fill and transposing tiles with several destinations."""
    _check_small(SMALL, SMALL_MIX, Parallel(2, 2, 1), Parallel(2, 2, 3))
    _check_small(ODD, ODD_MIX, Parallel(3, 1, 1), Parallel(4, 1, 2))
    _check_small(SMALL, SMALL_MIX, Parallel(2, 1, 1), Parallel(3, 2, 2, w_transposed=1))
    _check_small(WIDE, synth.MIX_GPT, Parallel(2, 1, 2), Parallel(4, 1, 4))


def test_shared_reads_eight_way_multicast(cuda):
    """Option share_reads on data-parallel scale-out: one read feeds up to eight replicas."""
    shared = dict(share_reads=1)
    plan = _check_small(SMALL, SMALL_MIX, Parallel(1, 1, 4), Parallel(1, 1, 8), opts=shared)
    assert all(b.n_dst == 8 for b in plan.boxes())
    _check_small(WIDE, synth.MIX_GPT, Parallel(2, 1, 2), Parallel(2, 1, 12), opts=shared)
    _check_small(ODD, ODD_MIX, Parallel(3, 1, 2), Parallel(4, 1, 5, w_transposed=1), opts=shared)
    plan = _check_small(SMALL, SMALL_MIX, Parallel(1, 1, 4), Parallel(1, 1, 8), opts=dict(share_reads=1, max_multicast=3))
    assert sorted({b.n_dst for b in plan.boxes()}) == [2, 3]           # 8 replicas as 3 + 3 + 2


def test_multicast_to_the_largest_replica_count(cuda):
    """One source replica copied to 128 (and, with two tensor-parallel ranks, 2 x 64) new replicas: with max_multicast at its
    limit every piece is one move with 128 (64) destinations, with 5 the replicas are served in groups of 5 and a rest."""
    plan = _check_small(SMALL, SMALL_MIX, Parallel(1, 1, 1), Parallel(1, 1, 128), opts=dict(max_multicast=128))
    assert {b.n_dst for b in plan.boxes()} == {128} and plan.stats()["bytes_written"] == 128 * plan.stats()["bytes_read"]
    plan = _check_small(SMALL, SMALL_MIX, Parallel(2, 1, 1), Parallel(2, 1, 64, w_transposed=1), opts=dict(max_multicast=128))
    assert {(b.n_dst, b.dst_rank_stride) for b in plan.boxes()} == {(64, 2)}
    plan = _check_small(SMALL, SMALL_MIX, Parallel(1, 1, 1), Parallel(1, 1, 128), opts=dict(max_multicast=5))
    assert sorted({b.n_dst for b in plan.boxes()}) == [3, 5]


DEEP = Model(n_layers=24, hidden=64, n_heads=4, ffn=256, vocab_true=512, max_pos=32)


@pytest.mark.parametrize("opts", [None, dict(pack_bytes=1), dict(pack_bytes=512), dict(tile_bytes=4096, pack_bytes=4096),
                                  dict(tile_bytes=65536, pack_bytes=65536)])
def test_short_moves_packed_into_shared_tiles(cuda, opts):
    """Biases and LayerNorm vectors share PACK tiles (up to 64 moves per tile, each with its own source and destination
    offset): single and replicated destinations, more moves per destination than one tile takes, every pack limit from
    none to the whole tile."""
    plan = _check_small(WIDE, synth.MIX_GPT, Parallel(4, 1, 1), Parallel(2, 2, 3), opts=opts)
    packs = [t for t in plan.tiles() if t.kind == tpx.binding.TILE_PACK]
    assert bool(packs) == (opts != dict(pack_bytes=1)) and {t.n_dst for t in packs} <= {1, 3}
    plan = _check_small(DEEP, synth.MIX_GPT, Parallel(2, 1, 1), Parallel(4, 1, 2), opts=opts)
    packs = [t for t in plan.tiles() if t.kind == tpx.binding.TILE_PACK]
    if opts != dict(pack_bytes=1):
        assert len(packs) > 8 and {t.n_dst for t in packs} == {2} and (opts is not None or max(t.n_seg for t in packs) == 64)
    _check_small(ODD, ODD_MIX, Parallel(3, 1, 2), Parallel(4, 1, 1, w_transposed=1), opts=opts)


MID = Model(n_layers=2, hidden=512, n_heads=8, ffn=2048, vocab_true=4096, max_pos=64)
TWELVE = Model(n_layers=2, hidden=192, n_heads=12, ffn=768, vocab_true=1536, max_pos=16)


@pytest.mark.parametrize("src,dst", [(Parallel(3, 1, 1), Parallel(4, 1, 1)), (Parallel(4, 1, 1), Parallel(3, 2, 1)),
                                     (Parallel(6, 1, 1), Parallel(4, 1, 2)), (Parallel(12, 1, 1), Parallel(2, 1, 1)),
                                     (Parallel(6, 2, 1), Parallel(4, 1, 1, qkv_layout=1))])
def test_merges_of_unequal_column_blocks(cuda, src, dst):
    """Thirds into quarters and the like: a new row of a row-parallel weight is made of column blocks of different widths,
    merged inside the tile (every segment with its own width), also as a multicast move."""
    print("case", src, dst, flush=True)
    plan = _check_small(TWELVE, synth.MIX_GPT, src, dst, seed=31, opts=dict(tile_bytes=16384))
    merges = [t for t in plan.tiles() if t.kind == tpx.binding.TILE_MERGE]
    if src.T % dst.T == 0:         # 12 -> 2: six equal blocks per row
        assert merges and all(t.seg_units * t.n_seg == t.run_units for t in merges)
    else:
        assert any(t.seg_units == 0 for t in merges)



@pytest.mark.parametrize("src,dst", [
    (Parallel(2, 1, 1), Parallel(4, 1, 1, w_transposed=1)),
    (Parallel(4, 1, 1, w_transposed=1, qkv_layout=1), Parallel(2, 2, 1)),
    (Parallel(2, 1, 1, w_transposed=1), Parallel(2, 1, 2, qkv_layout=1)),
    (Parallel(1, 1, 1), Parallel(8, 1, 1, w_transposed=1, qkv_layout=1)),
])
def test_transposed_storage_mid_size(cuda, src, dst):
    """[in, out] weight storage on one side: full 64 KiB blocks (512 x 64 bf16, 256 x 64 fp32) are transposed in one shot
    through LDS, edges take the general path; compared byte for byte with the oracle."""
    print("case", src, dst, flush=True)
    plan = _check_small(MID, synth.MIX_GPT, src, dst, seed=23)
    kinds = {b.kind for b in plan.boxes()}
    assert 2 in kinds        # TPX_BOX_TRANSPOSE


@pytest.mark.parametrize("chunk", [0, 1, 3, 8, 100])
@pytest.mark.parametrize("streams", [1, 2, 3, 4, 7, 8, 64, 1000])
def test_tile_order_streams(cuda, streams, chunk):
    """Any tile order gives the same bytes: streams that do or do not divide the tile count or the 8 XCDs, more streams
    than tiles, XCD-aware runs of any length (the surplus workgroups of the rounded-up grid exit)."""
    print("streams", streams, "chunk", chunk, flush=True)
    tpx.tpx_set_option("streams", streams)
    tpx.tpx_set_option("chunk", chunk)
    try:
        plan = _check_small(WIDE, synth.MIX_GPT, Parallel(4, 1, 1), Parallel(2, 2, 1), opts=dict(tile_bytes=8192))
        assert plan.num_tiles() % 7 != 0 or plan.num_tiles() % 64 != 0
        _check_small(SMALL, SMALL_MIX, Parallel(2, 1, 1), Parallel(1, 1, 1), opts=dict(tile_bytes=8192))
        _check_small(SMALL, SMALL_MIX, Parallel(2, 2, 1), Parallel(2, 2, 3), opts=dict(tile_bytes=4096))      # mixed plan: one stream
    finally:
        tpx.tpx_set_option("streams", 4)
        tpx.tpx_set_option("chunk", 0)


@pytest.mark.parametrize("occupancy", [1, 2, 3, 16])
def test_occupancy_cap(cuda, occupancy):
    """Workgroups per CU are capped through the LDS request; the bytes moved do not depend on it (copy, merge and
    transposing tiles, default 64 KiB tiles and 512-thread workgroups)."""
    tpx.tpx_set_option("occupancy", occupancy)
    try:
        _check_small(MID, synth.MIX_GPT, Parallel(4, 1, 1), Parallel(2, 2, 1), seed=23, opts=dict(tile_bytes=65536))
        _check_small(MID, synth.MIX_GPT, Parallel(2, 1, 1), Parallel(4, 1, 1, w_transposed=1), seed=23)
    finally:
        tpx.tpx_set_option("occupancy", 0)


def test_execute_inside_a_hip_graph(cuda):
    """After tpx_prepare, tpx_execute is a single kernel launch on the caller's stream, so it can be captured
    in a HIP graph and replayed; every replay (with the program's own work in between) must reproduce the
    eager result for the data then in the source buffers."""
    model, mix = WIDE, synth.MIX_GPT
    a, b = Parallel(2, 2, 1), Parallel(4, 1, 2)
    plan = plan_for(model, a, b)
    src = [x.cuda() for x in H.make_src_bufs(model, a, 9, mix)]
    dst = [G.alloc(plan.buffer_bytes(1, r), H.POISON) for r in range(b.n_ranks)]
    ws = G.alloc(plan.workspace_bytes())
    side = torch.cuda.Stream()
    plan.prepare(ws.data_ptr(), side.cuda_stream)
    sp, dp = [x.data_ptr() for x in src], [x.data_ptr() for x in dst]
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        plan.execute(sp, dp, ws.data_ptr(), torch.cuda.current_stream().cuda_stream)
    for seed in (9, 10, 11):
        fresh = H.make_src_bufs(model, a, seed, mix)
        for x, y in zip(src, fresh):
            x.copy_(y)
        for d in dst:
            d.fill_(H.POISON)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = oreshard.reshard(model, a, b, H.np_bufs(fresh))
        for r in range(b.n_ranks):
            assert np.array_equal(dst[r].cpu().numpy(), want[r]), (seed, r)
