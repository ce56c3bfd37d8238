"""TEST INFRASTRUCTURE ONLY - the CPU oracle's statement of the model-state layout.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; the product (the HIP library and its Python binding) never does,
and this package never imports the product.

What is described here (paper section 4.1, equation 1): a job's state is a
parallelizable tensor collection PTC = (T, sigma, phi, alpha):
  * T      the state tensors of a GPT-style model (every parameter tensor has
           one tensor per state kind: weight, optimizer copies);
  * sigma  slicing (tensor parallelism): which axis of a tensor is cut into
           `T` equal parts, or none (replicated on every tensor-parallel rank);
  * phi    partitioning: a layer's tensors belong to the pipeline stage that
           owns the layer; every data-parallel replica holds a full copy, except
           for state kinds marked as sharded over the replicas (sharded data
           parallelism: replica d keeps the d-th chunk of each of its tensors);
  * alpha  allocation: sub-collection (t, p, d) lives in rank buffer
           t + T*(d + D*p).
The paper leaves sigma/phi/alpha to the parallelizer (section 5.1: a JSON
object per GPU); the concrete Megatron-style rules below are this repository's
own written convention, implemented here independently of the planner.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import NamedTuple, Optional, Sequence

ALIGN = 256            # every stored tensor starts on a 256-byte boundary
POISON = 0xA5          # tests fill destination buffers with this byte first

# name index -> (name, per-layer?)
NAMES = (
    ("word_embeddings.weight", False),
    ("position_embeddings.weight", False),
    ("input_layernorm.weight", True),
    ("input_layernorm.bias", True),
    ("attention.query_key_value.weight", True),
    ("attention.query_key_value.bias", True),
    ("attention.dense.weight", True),
    ("attention.dense.bias", True),
    ("post_attention_layernorm.weight", True),
    ("post_attention_layernorm.bias", True),
    ("mlp.dense_h_to_4h.weight", True),
    ("mlp.dense_h_to_4h.bias", True),
    ("mlp.dense_4h_to_h.weight", True),
    ("mlp.dense_4h_to_h.bias", True),
    ("final_layernorm.weight", False),
    ("final_layernorm.bias", False),
)
N_LAYER_NAMES = 12
(WORD_EMB, POS_EMB, LN1_W, LN1_B, QKV_W, QKV_B, DENSE_W, DENSE_B, LN2_W, LN2_B,
 FC1_W, FC1_B, FC2_W, FC2_B, LNF_W, LNF_B) = range(16)


@dataclass(frozen=True)
class Model:
    n_layers: int
    hidden: int
    n_heads: int
    ffn: int
    vocab_true: int
    max_pos: int = 1024
    vocab_divisor: int = 0              # 0: vocab must divide by T; else pad to a multiple of divisor*T
    state_elem_bytes: tuple = (2, 4, 4, 4)
    tied_head: bool = False             # copy of word embeddings on the last stage when P > 1

    @property
    def head_dim(self) -> int:
        return self.hidden // self.n_heads

    @property
    def n_tensors(self) -> int:
        return N_LAYER_NAMES * self.n_layers + 4


@dataclass(frozen=True)
class Parallel:
    T: int
    P: int
    D: int
    stage_first_layer: Optional[tuple] = None   # P+1 ascending boundaries; None = even split
    qkv_layout: int = 0                         # 0 head-major [a,3,d,*]; 1 qkv-major [3,a,d,*]
    w_transposed: int = 0                       # 1: 2-D weights stored [in, out] instead of [out, in]
    shard_kinds: int = 0                        # bit k set: state kind k is sharded over the D replicas
    layer_stage: Optional[tuple] = None         # stage of every layer (any map, e.g. interleaved chunks); overrides stage_first_layer

    @property
    def n_ranks(self) -> int:
        return self.T * self.P * self.D


class Entry(NamedTuple):
    """One stored tensor block in a rank buffer (same fields as synth.ShardDesc plus name, layer)."""
    tensor_id: int
    kind: int
    elem_bytes: int
    offset: int
    full_shape: tuple
    lo: tuple
    hi: tuple
    perm: tuple
    name: int
    layer: int      # -1 for global tensors


def tensor_id(name: int, layer: int) -> int:
    if not NAMES[name][1]:
        return name if name < 2 else 2 + (name - LNF_W)          # 0,1 embeddings; 2,3 final LN
    return 4 + layer * N_LAYER_NAMES + (name - LN1_W)


def vocab_padded(model: Model, T: int) -> int:
    if model.vocab_divisor == 0:
        if model.vocab_true % T:
            raise ValueError("vocab not divisible by T and no padding divisor given")
        return model.vocab_true
    m = model.vocab_divisor * T
    return -(-model.vocab_true // m) * m


def check(model: Model, par: Parallel) -> None:
    if min(par.T, par.P, par.D) < 1:
        raise ValueError("degrees must be >= 1")
    if model.hidden % model.n_heads:
        raise ValueError("hidden must be a multiple of n_heads")
    if model.n_heads % par.T or model.ffn % par.T or model.hidden % par.T:
        raise ValueError("heads / ffn / hidden not divisible by T")
    vocab_padded(model, par.T)
    if par.layer_stage is not None:
        if len(par.layer_stage) != model.n_layers or any(not 0 <= p < par.P for p in par.layer_stage):
            raise ValueError("layer_stage needs one stage index below P per layer")
    else:
        stage_bounds(model, par)
    if par.shard_kinds >> len(model.state_elem_bytes):
        raise ValueError("shard_kinds names a state kind the model does not have")


def stage_bounds(model: Model, par: Parallel) -> tuple:
    if par.stage_first_layer is None:
        if model.n_layers % par.P:
            raise ValueError("layers not divisible by P")
        per = model.n_layers // par.P
        return tuple(p * per for p in range(par.P + 1))
    b = tuple(par.stage_first_layer)
    if len(b) != par.P + 1 or b[0] != 0 or b[-1] != model.n_layers or any(b[i] > b[i + 1] for i in range(par.P)):
        raise ValueError("bad stage map")
    return b


def rank_of(par: Parallel, t: int, p: int, d: int) -> int:
    return t + par.T * (d + par.D * p)


def coords_of(par: Parallel, rank: int) -> tuple:
    t = rank % par.T
    d = (rank // par.T) % par.D
    p = rank // (par.T * par.D)
    return t, p, d


def canonical(model: Model, par: Parallel, name: int):
    """(full canonical shape, split axis or None, storage perm) of a parameter tensor."""
    h, a, dh, f = model.hidden, model.n_heads, model.head_dim, model.ffn
    tr = par.w_transposed
    if name == WORD_EMB:
        return (vocab_padded(model, par.T), h), 0, (0, 1)
    if name == POS_EMB:
        return (model.max_pos, h), None, (0, 1)
    if name in (LN1_W, LN1_B, LN2_W, LN2_B, DENSE_B, FC2_B, LNF_W, LNF_B):
        return (h,), None, (0,)
    if name == QKV_W:
        out = (0, 1, 2) if par.qkv_layout == 0 else (1, 0, 2)
        return (a, 3, dh, h), 0, ((3,) + out if tr else out + (3,))
    if name == QKV_B:
        return (a, 3, dh), 0, ((0, 1, 2) if par.qkv_layout == 0 else (1, 0, 2))
    if name == DENSE_W:
        return (h, h), 1, ((1, 0) if tr else (0, 1))
    if name == FC1_W:
        return (f, h), 0, ((1, 0) if tr else (0, 1))
    if name == FC1_B:
        return (f,), 0, (0,)
    if name == FC2_W:
        return (h, f), 1, ((1, 0) if tr else (0, 1))
    raise ValueError(name)


def stage_tensors(model: Model, par: Parallel, p: int):
    """(name, layer) of every parameter tensor held by stage p, in packing order."""
    if par.layer_stage is not None:
        layers = [layer for layer in range(model.n_layers) if par.layer_stage[layer] == p]
    else:
        b = stage_bounds(model, par)
        layers = range(b[p], b[p + 1])
    out = []
    if p == 0:
        out += [(WORD_EMB, -1), (POS_EMB, -1)]
    for layer in layers:
        out += [(n, layer) for n in range(LN1_W, LN1_W + N_LAYER_NAMES)]
    if p == par.P - 1:
        out += [(LNF_W, -1), (LNF_B, -1)]
        if model.tied_head and par.P > 1:
            out += [(WORD_EMB, -1)]
    return out


def shard_range(full_shape: Sequence[int], axis, T: int, t: int):
    lo = [0] * len(full_shape)
    hi = list(full_shape)
    if axis is not None:
        n = full_shape[axis] // T
        lo[axis], hi[axis] = t * n, (t + 1) * n
    return tuple(lo), tuple(hi)


def replica_range(lo, hi, perm, D: int, d: int):
    """Sharded data parallelism: of the block [lo, hi) that a (t, p) share holds, replica d keeps chunk d
    along the block's outermost stored axis (perm[0]), chunks of ceil(extent / D) - the last ones may be
    short or empty.  Returns (lo, hi) of the chunk, or None if it is empty."""
    ax = perm[0]
    n = hi[ax] - lo[ax]
    c = -(-n // D)
    a, b = min(n, d * c), min(n, (d + 1) * c)
    if a == b:
        return None
    lo2, hi2 = list(lo), list(hi)
    lo2[ax], hi2[ax] = lo[ax] + a, lo[ax] + b
    return tuple(lo2), tuple(hi2)


def _numel(lo, hi) -> int:
    n = 1
    for l, u in zip(lo, hi):
        n *= u - l
    return n


def rank_manifest(model: Model, par: Parallel, rank: int):
    """(entries, buffer_bytes) of one rank buffer: state-kind-major arenas, inside
    each the stage's tensors in packing order, each aligned to ALIGN bytes."""
    check(model, par)
    t, p, d = coords_of(par, rank)
    entries = []
    off = 0
    for kind, eb in enumerate(model.state_elem_bytes):
        for name, layer in stage_tensors(model, par, p):
            full, axis, perm = canonical(model, par, name)
            lo, hi = shard_range(full, axis, par.T, t)
            if (par.shard_kinds >> kind) & 1:
                chunk = replica_range(lo, hi, perm, par.D, d)
                if chunk is None:
                    continue            # this replica holds nothing of the tensor
                lo, hi = chunk
            off = -(-off // ALIGN) * ALIGN
            entries.append(Entry(tensor_id(name, layer), kind, eb, off, full, lo, hi, perm, name, layer))
            off += _numel(lo, hi) * eb
    return entries, -(-off // ALIGN) * ALIGN


def n_params(model: Model, T: int = 1) -> int:
    """Closed form of the parameter count (with the vocab padding of degree T)."""
    h, f = model.hidden, model.ffn
    per_layer = 3 * h * h + 3 * h + h * h + h + 2 * f * h + f + h + 4 * h
    return model.n_layers * per_layer + vocab_padded(model, T) * h + model.max_pos * h + 2 * h
