"""Shared test helpers: the benchmark configurations, synthetic buffers built
from the oracle's layout, and conversions between the oracle's manifest entries
and the input generator's block descriptions."""
from __future__ import annotations

import torch

import synth
from oracle import spec
from oracle.spec import Model, Parallel

SRC_GAP = 0x5A     # byte in alignment gaps of source buffers
POISON = spec.POISON

TINY = Model(n_layers=2, hidden=256, n_heads=4, ffn=1024, vocab_true=1024, max_pos=1024,
             state_elem_bytes=(4, 4, 4))
GPT_1_3B = Model(n_layers=24, hidden=2048, n_heads=16, ffn=8192, vocab_true=50304)
GPT_2_7B = Model(n_layers=32, hidden=2560, n_heads=32, ffn=10240, vocab_true=50304)
GPT_6_7B = Model(n_layers=32, hidden=4096, n_heads=32, ffn=16384, vocab_true=50304)
GPT_ODD = Model(n_layers=24, hidden=3072, n_heads=24, ffn=12288, vocab_true=50257, vocab_divisor=128)

# the five workloads: (model, source config, destination config, state mix, seed)
CONFIGS = {
    1: (TINY, Parallel(2, 1, 1), Parallel(4, 2, 1), synth.MIX_TINY, 1),
    2: (GPT_1_3B, Parallel(4, 2, 1), Parallel(2, 4, 1), synth.MIX_GPT, 2),
    3: (GPT_2_7B, Parallel(4, 4, 2), Parallel(2, 4, 1, stage_first_layer=(0, 7, 16, 25, 32)), synth.MIX_GPT, 3),
    4: (GPT_6_7B, Parallel(8, 1, 1), Parallel(1, 8, 1), synth.MIX_GPT, 4),
    5: (GPT_ODD, Parallel(3, 1, 1), Parallel(4, 1, 1), synth.MIX_GPT, 5),
}
DATASET_CFG = dict(n_samples=10 ** 8, global_batch=768, D_src=6, D_dst=4, steps_done=65000, seed=6)


def scaled(model: Model, **kw) -> Model:
    d = dict(model.__dict__)
    d.update(kw)
    return Model(**d)


def desc_of(e) -> synth.ShardDesc:
    return synth.ShardDesc(e.tensor_id, e.kind, e.elem_bytes, e.offset, tuple(e.full_shape),
                           tuple(e.lo), tuple(e.hi), tuple(e.perm))


def manifest_descs(model, par):
    """[(descs, nbytes)] per rank, from the oracle's layout."""
    out = []
    for r in range(par.n_ranks):
        entries, n = spec.rank_manifest(model, par, r)
        out.append(([desc_of(e) for e in entries], n))
    return out


def make_src_bufs(model, par, seed, mix, device="cpu"):
    bufs = []
    for descs, n in manifest_descs(model, par):
        b = torch.full((n,), SRC_GAP, dtype=torch.uint8, device=device)
        synth.fill_buffer(b, descs, seed, mix)
        bufs.append(b)
    return bufs


def _zero_rule(model, src_par):
    """Rows of the word embedding at or beyond the source's padded vocabulary are zero."""
    v_src = spec.vocab_padded(model, src_par.T)

    def rule(d):
        return v_src if d.tensor_id == spec.tensor_id(spec.WORD_EMB, -1) else None
    return rule


def closed_form_dst_bufs(model, src_par, dst_par, seed, mix, device="cpu"):
    """What the destination buffers must hold, straight from the value function."""
    bufs = []
    for descs, n in manifest_descs(model, dst_par):
        b = torch.full((n,), POISON, dtype=torch.uint8, device=device)
        synth.fill_buffer(b, descs, seed, mix, zero_from_row=_zero_rule(model, src_par))
        bufs.append(b)
    return bufs


def closed_form_mismatches(bufs, model, src_par, dst_par, seed, mix) -> int:
    bad = 0
    for b, (descs, n) in zip(bufs, manifest_descs(model, dst_par)):
        assert b.numel() == n
        bad += synth.count_mismatch(b, descs, seed, mix, zero_from_row=_zero_rule(model, src_par))
    return bad


def gaps_untouched(buf: torch.Tensor, descs, fill: int) -> bool:
    """True if every byte of buf outside the described blocks still equals `fill`."""
    pos = 0
    for d in sorted(descs, key=lambda d: d.offset):
        if pos < d.offset and not bool((buf[pos:d.offset] == fill).all()):
            return False
        pos = d.offset + d.nbytes
    return bool((buf[pos:] == fill).all())


def np_bufs(bufs):
    return [b.cpu().numpy() for b in bufs]
