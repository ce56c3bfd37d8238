"""tpx_execute_static: the entry point for callers that cannot allocate (the plan tables sit in a static
device array of the library instead of a caller-supplied workspace).  Through the C ABI, bit for bit
against tpx_execute and against the CPU oracle: a larger job first, then a smaller one, then the first
again, all through the one shared array."""
import numpy as np
import pytest
import torch

import paper_2312_05181_amd as tpx
import paper_2312_05181_amd.binding as B
import synth
from oracle import reshard as oreshard
from oracle.spec import Model, Parallel
from tests import gpu_util as G
from tests import helpers as H
from tests.test_planner import SMALL, SMALL_MIX, WIDE, plan_for

MID = Model(n_layers=2, hidden=512, n_heads=8, ffn=2048, vocab_true=4096, max_pos=64)


def _both_ways(model, mix, a, b, seed):
    """(outputs of tpx_execute, outputs of tpx_execute_static, the oracle's buffers) for one reshard."""
    src_cpu = H.make_src_bufs(model, a, seed, mix)
    want = oreshard.reshard(model, a, b, H.np_bufs(src_cpu))
    plan = plan_for(model, a, b)
    assert plan.workspace_bytes() <= B.TPX_STATIC_WORKSPACE_BYTES
    src = [x.cuda() for x in src_cpu]
    ref, _ = G.execute(plan, src)
    got = [G.alloc(plan.buffer_bytes(1, r), H.POISON) for r in range(b.n_ranks)]
    torch.cuda.synchronize()
    return plan, src, ref, got, want


def _run_static(plan, src, got):
    before = torch.cuda.memory_allocated()
    tpx.tpx_execute_static(plan, [x.data_ptr() for x in src], [x.data_ptr() for x in got],
                           torch.cuda.current_stream().cuda_stream)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()


def _same(got, ref, want):
    for r, (g, x, w) in enumerate(zip(got, ref, want)):
        assert torch.equal(g, x), f"rank {r}: differs from tpx_execute"
        assert np.array_equal(g.cpu().numpy(), w), f"rank {r}: differs from the oracle"


@pytest.mark.gpu
def test_static_tables_two_calls_in_a_row_second_smaller(cuda):
    print("static tables: larger job", flush=True)
    big = _both_ways(MID, synth.MIX_GPT, Parallel(2, 1, 1), Parallel(4, 2, 1, w_transposed=1), 23)
    print("static tables: smaller job", flush=True)
    small = _both_ways(SMALL, SMALL_MIX, Parallel(2, 1, 1), Parallel(1, 2, 1), 5)
    assert small[0].workspace_bytes() < big[0].workspace_bytes()
    assert small[0].stats()["bytes_written"] < big[0].stats()["bytes_written"]
    for plan, src, ref, got, want in (big, small):       # the second call finds the first one's tables in the array
        _run_static(plan, src, got)
        _same(got, ref, want)
    print("static tables: the larger job again, then twice without an upload in between", flush=True)
    plan, src, ref, got, want = big
    for _ in range(2):
        for g in got:
            g.fill_(H.POISON)
        _run_static(plan, src, got)
        _same(got, ref, want)


@pytest.mark.gpu
def test_static_tables_merge_multicast_and_fill_tiles(cuda):
    plan, src, ref, got, want = _both_ways(WIDE, synth.MIX_GPT, Parallel(4, 1, 1), Parallel(2, 1, 3), 9)
    _run_static(plan, src, got)
    _same(got, ref, want)


@pytest.mark.gpu
def test_static_tables_argument_errors(cuda):
    plan = plan_for(SMALL, Parallel(2, 1, 1), Parallel(1, 1, 1))
    src = [G.alloc(plan.buffer_bytes(0, r), 0) for r in range(2)]
    dst = [G.alloc(plan.buffer_bytes(1, 0), H.POISON)]
    with pytest.raises(tpx.TpxError) as err:
        tpx.tpx_execute_static(plan, [src[0].data_ptr(), 0], [dst[0].data_ptr()])
    assert err.value.status == B.TPX_ERR_INVALID_ARG
    with pytest.raises(tpx.TpxError):
        tpx.tpx_execute_static(plan, [src[0].data_ptr() + 4, src[1].data_ptr()], [dst[0].data_ptr()])
    torch.cuda.synchronize()
    assert bool((dst[0] == H.POISON).all())


def test_plan_tables_beyond_the_static_array_are_refused():
    """Checked on the host before any GPU call: a layout-changing reshard of 128 heads x 32 layers, whose
    transposing moves enumerate (head, q/k/v) pairs into about 50,000 flat boxes."""
    model = Model(n_layers=32, hidden=1024, n_heads=128, ffn=1024, vocab_true=1024)
    plan = plan_for(model, Parallel(1, 1, 1), Parallel(1, 1, 1, qkv_layout=1, w_transposed=1))
    assert plan.workspace_bytes() > B.TPX_STATIC_WORKSPACE_BYTES
    n_src, n_dst = plan.num_buffers(0), plan.num_buffers(1)
    with pytest.raises(tpx.TpxError) as err:
        tpx.tpx_execute_static(plan, [256] * n_src, [256] * n_dst)       # never dereferenced
    assert err.value.status == B.TPX_ERR_TOO_LARGE and "TPX_STATIC_WORKSPACE_BYTES" in str(err.value)
