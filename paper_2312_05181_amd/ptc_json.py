"""Importer for parallelization configurations given as JSON (paper section 5.1: a list with one object per
GPU that follows the structure of the model that GPU hosts, tensors as leaves).  Marshalling only: it turns
the two JSON documents into the manifests tpx_plan_ptc takes.

A leaf is an object with
    "full_shape": [..]          shape of the whole tensor
    "offset":     [..]          where this GPU's block starts in the whole tensor (default: zeros)
    "shape":      [..]          shape of the block this GPU stores (default: full_shape)
    "dtype":      "bfloat16" | "float16" | "float32" | "float64" | "int8" | "uint8" | "int16" | "int32" | "int64"
    "perm":       [..]          optional storage order (stored axis i = tensor axis perm[i])
Every other object is a module; a tensor's identity is its path ("/transformer/h/0/attn/c_attn/weight"),
the same on both sides.  Where a block sits in its rank buffer is left to the library (offset None: it packs
a rank's blocks in document order; the plan's manifest tells where).
"""
from __future__ import annotations

import json
from collections import namedtuple

Block = namedtuple("Block", "tensor_id kind elem_bytes offset full_shape lo hi perm name layer path")

_BYTES = {"bfloat16": 2, "float16": 2, "float32": 4, "float64": 8, "int8": 1, "uint8": 1, "int16": 2, "int32": 4,
          "int64": 8}


def _leaves(node, path=""):
    if isinstance(node, dict) and "full_shape" in node:
        yield path, node
    elif isinstance(node, dict):
        for k, v in node.items():
            yield from _leaves(v, f"{path}/{k}")
    elif isinstance(node, list):
        for i, v in enumerate(node):
            yield from _leaves(v, f"{path}/{i}")
    else:
        raise ValueError(f"{path}: expected a module or a tensor leaf")


def manifests_from_json(src_text: str, dst_text: str):
    """-> (src_manifests, dst_manifests, names); names[tensor_id] = path.  The manifests are what tpx_plan_ptc takes."""
    docs = [json.loads(src_text), json.loads(dst_text)]
    for d in docs:
        if not isinstance(d, list):
            raise ValueError("top level must be a list with one object per GPU")
    names = sorted({p for d in docs for gpu in d for p, _ in _leaves(gpu)})
    ids = {p: i for i, p in enumerate(names)}
    out = []
    for d in docs:
        mans = []
        for gpu in d:
            blocks = []
            for path, leaf in _leaves(gpu):
                full = tuple(int(x) for x in leaf["full_shape"])
                lo = tuple(int(x) for x in leaf.get("offset", [0] * len(full)))
                shape = tuple(int(x) for x in leaf.get("shape", full))
                hi = tuple(a + b for a, b in zip(lo, shape))
                perm = tuple(int(x) for x in leaf.get("perm", range(len(full))))
                blocks.append(Block(ids[path], 0, _BYTES[leaf.get("dtype", "float32")], None, full, lo, hi, perm, 0, -1, path))
            mans.append(blocks)
        out.append(mans)
    return out[0], out[1], names
