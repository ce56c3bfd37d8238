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
from tests.test_planner import ODD, ODD_MIX, PAIRS, SMALL, SMALL_MIX, WIDE, mk, pk, plan_for

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
    tpx.tpx_set_option("tile_bytes", tile_bytes)
    try:
        plan = _check_small(WIDE, synth.MIX_GPT, src, dst)
        assert plan.num_tiles() > 100
    finally:
        tpx.tpx_set_option("tile_bytes", 131072)


@pytest.mark.parametrize("variant", [u | (n * 24) | (t << 5) for t in range(3) for n in range(2) for u in (2, 3, 4)])
def test_every_kernel_variant(cuda, variant):
    print("variant", variant, flush=True)
    tpx.tpx_set_option("variant", variant)
    tpx.tpx_set_option("tile_bytes", 16384)
    try:
        _check_small(WIDE, synth.MIX_GPT, Parallel(4, 1, 1), Parallel(2, 2, 1))
        _check_small(ODD, ODD_MIX, Parallel(3, 1, 1), Parallel(4, 1, 1))
    finally:
        tpx.tpx_set_option("variant", 0)
        tpx.tpx_set_option("tile_bytes", 131072)


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
    with pytest.raises(tpx.TpxError):
        tpx.tpx_execute(plan, [src[0].data_ptr(), 0], [dst[0].data_ptr()], ws.data_ptr())
    with pytest.raises(tpx.TpxError):
        tpx.tpx_execute(plan, [src[0].data_ptr() + 4, src[1].data_ptr()], [dst[0].data_ptr()], ws.data_ptr())
    with pytest.raises(tpx.TpxError):
        tpx.tpx_execute(plan, [s.data_ptr() for s in src], [dst[0].data_ptr()], ws.data_ptr() + 8)
    with pytest.raises(tpx.TpxError):
        tpx.tpx_execute(plan, [s.data_ptr() for s in src], [dst[0].data_ptr()], 0)
    torch.cuda.synchronize()


def test_recycled_workspace_moves_nothing_and_is_reported(cuda):
    """A workspace overwritten by another plan's tables since the upload: the launch must not follow them."""
    model, mix = SMALL, SMALL_MIX
    a, b = Parallel(2, 1, 1), Parallel(1, 2, 1)
    src_cpu = H.make_src_bufs(model, a, 3, mix)
    want = oreshard.reshard(model, a, b, H.np_bufs(src_cpu))
    src = [x.cuda() for x in src_cpu]
    first, other = plan_for(model, a, b), plan_for(model, a, Parallel(2, 2, 1))
    ws = G.alloc(max(first.workspace_bytes(), other.workspace_bytes()))
    stream = torch.cuda.current_stream().cuda_stream
    got, _ = G.execute(first, src, workspace=ws)
    first.workspace_check(ws.data_ptr(), stream)
    assert all(np.array_equal(g.cpu().numpy(), w) for g, w in zip(got, want))
    other.prepare(ws.data_ptr(), stream)                         # the other plan's tables now sit in ws
    other.workspace_check(ws.data_ptr(), stream)
    stale, _ = G.execute(first, src, workspace=ws)               # `first` still believes ws is its own
    with pytest.raises(tpx.TpxError) as err:
        first.workspace_check(ws.data_ptr(), stream)
    assert err.value.status == tpx.binding.TPX_ERR_STALE_WORKSPACE
    assert all(bool((x == H.POISON).all()) for x in stale)       # nothing was written
    ws.zero_()                                                   # garbage instead of any plan
    stale, _ = G.execute(first, src, workspace=ws)
    torch.cuda.synchronize()
    assert all(bool((x == H.POISON).all()) for x in stale)
    first.workspace_forget()                                     # told so, it uploads again
    got, _ = G.execute(first, src, workspace=ws)
    first.workspace_check(ws.data_ptr(), stream)
    assert all(np.array_equal(g.cpu().numpy(), w) for g, w in zip(got, want))


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
def _dataset_case(n, Bsz, D, D2, s, seed=6):
    Gord = synth.epoch_order(n, seed) if n else np.zeros(0, dtype=np.uint64)
    parts = ods.partition(Gord, Bsz, D)
    cur = ods.cursors_after(n, Bsz, D, s)
    want_parts, want_cur = ods.repartition(parts, cur, Bsz, D2)
    plan = tpx.tpx_plan_dataset(n, Bsz, D, D2, cur)
    assert plan.dst_cursors == want_cur
    src = [torch.from_numpy(p.view(np.uint8).copy()).cuda() if p.size else torch.empty(0, dtype=torch.uint8, device="cuda")
           for p in parts]
    got, _ = G.execute(plan, src)
    torch.cuda.synchronize()
    for j in range(D2):
        assert np.array_equal(got[j].cpu().numpy().view(np.uint64), want_parts[j]), j


@pytest.mark.parametrize("n,Bsz,D,D2,s", [(100, 24, 6, 4, 2), (101, 24, 4, 6, 3), (7, 12, 6, 4, 1), (0, 12, 2, 3, 0),
                                          (768 * 50 + 256, 768, 6, 4, 20), (100000, 768, 4, 6, 130), (1000, 48, 6, 6, 7)])
def test_dataset_small(cuda, n, Bsz, D, D2, s):
    print("dataset", n, Bsz, D, D2, s, flush=True)
    _dataset_case(n, Bsz, D, D2, s)


def test_dataset_full_size(cuda):
    c = H.DATASET_CFG
    print("dataset full size", c, flush=True)
    _dataset_case(c["n_samples"], c["global_batch"], c["D_src"], c["D_dst"], c["steps_done"], c["seed"])


# ---------------------------------------------------------------------------------------------
# the paper's own reconfigurations (sections 6.2, 6.3, 6.6, 6.8) at full size
# ---------------------------------------------------------------------------------------------
def _paper_pairs():
    import bench
    return [k for k in bench.PAPER_PAIRS if not k.startswith("gpt6.7b") and not k.startswith("gpt2.7b_(4,2,1)->(4,4")] + \
        list(bench.SHARDED_PAIRS)          # plus the sharded-optimizer-state reshards, checked the same way


@pytest.mark.parametrize("name", _paper_pairs())
def test_paper_reconfiguration_pairs(cuda, name):
    """Data-, pipeline- and tensor-parallel changes, redeployment and the elastic-scaling sequence of the
    paper's evaluation: every destination tensor equals its closed-form contents, gaps stay untouched, and
    replicated destinations are written from a single read (multicast moves)."""
    import bench
    mk_, s_, d_, _, seed = bench.WORKLOADS[name]
    print("pair", name, flush=True)
    model = Model(mk_["n_layers"], mk_["hidden"], mk_["n_heads"], mk_["ffn"], mk_["vocab_true"], mk_.get("max_pos", 1024),
                  mk_.get("vocab_divisor", 0), tuple(mk_["state_elem_bytes"]))
    src = Parallel(s_["T"], s_["P"], s_["D"], s_.get("stage_first_layer"), shard_kinds=s_.get("shard_kinds", 0),
                   layer_stage=s_.get("layer_stage"))
    dst = Parallel(d_["T"], d_["P"], d_["D"], d_.get("stage_first_layer"), shard_kinds=d_.get("shard_kinds", 0),
                   layer_stage=d_.get("layer_stage"))
    mix = synth.MIX_GPT
    plan = plan_for(model, src, dst)
    st = plan.stats()
    if src.D == 1 and dst.D > 1 and src.T == dst.T and src.P == dst.P:
        assert st["bytes_read"] * dst.D == st["bytes_written"]        # read once, written D' times
    assert st["bytes_read"] <= st["bytes_written"]
    src_gpu = []
    for descs, n in H.manifest_descs(model, src):
        b = G.alloc(n, H.SRC_GAP)
        synth.fill_buffer(b, descs, seed, mix)
        src_gpu.append(b)
    got, _ = G.execute(plan, src_gpu)
    torch.cuda.synchronize()
    assert H.closed_form_mismatches(got, model, src, dst, seed, mix) == 0
    for b, (descs, n) in zip(got, H.manifest_descs(model, dst)):
        assert H.gaps_untouched(b, descs, H.POISON)
    del got, src_gpu
    torch.cuda.empty_cache()


def test_shared_reads_full_size(cuda):
    """BERT-large-shape (1,1,4) -> (1,1,8) with share_reads: one 8-way multicast move per piece, every replica
    complete (closed form), gaps untouched, one fifth of the reads of the locality plan."""
    import bench
    mk_, s_, d_, _, seed = bench.WORKLOADS["bert-large_(1,1,4)->(1,1,8)"]
    model = Model(mk_["n_layers"], mk_["hidden"], mk_["n_heads"], mk_["ffn"], mk_["vocab_true"], mk_.get("max_pos", 1024),
                  mk_.get("vocab_divisor", 0), tuple(mk_["state_elem_bytes"]))
    src, dst = Parallel(1, 1, 4), Parallel(1, 1, 8)
    local = plan_for(model, src, dst).stats()
    tpx.tpx_set_option("share_reads", 1)
    try:
        plan = plan_for(model, src, dst)
    finally:
        tpx.tpx_set_option("share_reads", 0)
    st = plan.stats()
    assert st["bytes_written"] == local["bytes_written"] == 8 * st["bytes_read"] and local["bytes_read"] == 5 * st["bytes_read"]
    src_gpu = []
    for descs, n in H.manifest_descs(model, src):
        b = G.alloc(n, H.SRC_GAP)
        synth.fill_buffer(b, descs, seed, synth.MIX_GPT)
        src_gpu.append(b)
    got, _ = G.execute(plan, src_gpu)
    torch.cuda.synchronize()
    assert H.closed_form_mismatches(got, model, src, dst, seed, synth.MIX_GPT) == 0
    for b, (descs, n) in zip(got, H.manifest_descs(model, dst)):
        assert H.gaps_untouched(b, descs, H.POISON)
    del got, src_gpu
    torch.cuda.empty_cache()


def test_multicast_small(cuda):
    """Replicated destinations on odd-sized models: copy, fill and transposing tiles with several destinations."""
    _check_small(SMALL, SMALL_MIX, Parallel(2, 2, 1), Parallel(2, 2, 3))
    _check_small(ODD, ODD_MIX, Parallel(3, 1, 1), Parallel(4, 1, 2))
    _check_small(SMALL, SMALL_MIX, Parallel(2, 1, 1), Parallel(3, 2, 2, w_transposed=1))
    _check_small(WIDE, synth.MIX_GPT, Parallel(2, 1, 2), Parallel(4, 1, 4))


def test_shared_reads_eight_way_multicast(cuda):
    """Option share_reads on data-parallel scale-out: one read feeds up to eight replicas."""
    tpx.tpx_set_option("share_reads", 1)
    try:
        plan = _check_small(SMALL, SMALL_MIX, Parallel(1, 1, 4), Parallel(1, 1, 8))
        assert all(b.n_dst == 8 for b in plan.boxes())
        _check_small(WIDE, synth.MIX_GPT, Parallel(2, 1, 2), Parallel(2, 1, 12))
        _check_small(ODD, ODD_MIX, Parallel(3, 1, 2), Parallel(4, 1, 5, w_transposed=1))
    finally:
        tpx.tpx_set_option("share_reads", 0)


MID = Model(n_layers=2, hidden=512, n_heads=8, ffn=2048, vocab_true=4096, max_pos=64)


@pytest.mark.parametrize("src,dst", [
    (Parallel(2, 1, 1), Parallel(4, 1, 1, w_transposed=1)),
    (Parallel(4, 1, 1, w_transposed=1, qkv_layout=1), Parallel(2, 2, 1)),
    (Parallel(2, 1, 1, w_transposed=1), Parallel(2, 1, 2, qkv_layout=1)),
    (Parallel(1, 1, 1), Parallel(8, 1, 1, w_transposed=1, qkv_layout=1)),
])
def test_transposed_storage_mid_size(cuda, src, dst):
    """[in, out] weight storage on one side: full 128 x 128 (bf16) and 64 x 64 (fp32) sub-tiles take the
    vectorised LDS path, edges the element path; compared byte for byte with the oracle."""
    print("case", src, dst, flush=True)
    plan = _check_small(MID, synth.MIX_GPT, src, dst, seed=23)
    kinds = {b.kind for b in plan.boxes()}
    assert 2 in kinds        # TPX_BOX_TRANSPOSE


@pytest.mark.parametrize("streams", [1, 3, 4, 7, 8, 64, 1000])
def test_tile_order_streams(cuda, streams):
    """Any tile order gives the same bytes, also when the tile count is not a multiple of the stream count
    or smaller than it (the surplus workgroups exit)."""
    print("streams", streams, flush=True)
    tpx.tpx_set_option("streams", streams)
    tpx.tpx_set_option("tile_bytes", 8192)
    try:
        plan = _check_small(WIDE, synth.MIX_GPT, Parallel(4, 1, 1), Parallel(2, 2, 1))
        assert plan.num_tiles() % 7 != 0 or plan.num_tiles() % 64 != 0
        _check_small(SMALL, SMALL_MIX, Parallel(2, 1, 1), Parallel(1, 1, 1))
    finally:
        tpx.tpx_set_option("streams", 4)
        tpx.tpx_set_option("tile_bytes", 131072)


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
