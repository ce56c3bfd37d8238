"""TEST INFRASTRUCTURE ONLY - CPU oracle of the dataset-state transformation.

The paper (sections 2.2 and 5.2) fixes requirements, not a formula: every
sample is consumed exactly once per epoch, the order in which samples are
consumed does not change when the data-parallel degree changes, and the global
batch size stays constant; each data partition has its own index.  The reading
implemented here:

  * G[0..N) is the epoch's global order of sample ids, B the global batch,
    D the number of replicas, b = B / D the local batch;
  * at step k replica j consumes G[k*B + j*b : k*B + (j+1)*b] (clipped to N);
    partition j is the concatenation of those chunks over k, i.e. the entries
    G[p] with (p mod B) div b == j, in increasing p;
  * the cursor of partition j counts its consumed entries; after s whole steps
    it is min(len(partition j), s*b).

Repartitioning rebuilds G from the old partitions by the inverse of that rule
and applies the rule again with the new degree.
"""
from __future__ import annotations

import numpy as np


def _owner(n: int, B: int, D: int) -> np.ndarray:
    if B % D:
        raise ValueError("global batch must be divisible by the replica count")
    p = np.arange(n, dtype=np.int64)
    return (p % B) // (B // D)


def partition(G: np.ndarray, B: int, D: int) -> list:
    """Per-replica index arrays of global order G."""
    own = _owner(len(G), B, D)
    return [G[own == j] for j in range(D)]


def cursors_after(n: int, B: int, D: int, s: int) -> list:
    own = _owner(n, B, D)
    b = B // D
    return [int(min(np.count_nonzero(own == j), s * b)) for j in range(D)]


def global_order(parts: list, B: int) -> np.ndarray:
    """Inverse of partition()."""
    D = len(parts)
    n = sum(len(p) for p in parts)
    own = _owner(n, B, D)
    G = np.empty((n,) + parts[0].shape[1:], dtype=parts[0].dtype)   # an entry may be a row (e.g. an (offset, length) pair)
    for j in range(D):
        if np.count_nonzero(own == j) != len(parts[j]):
            raise ValueError("partition sizes are not those of a consistent partitioning")
        G[own == j] = parts[j]
    return G


def steps_done(sizes: list, cursors: list, B: int) -> int:
    """The smallest step count s with cursors[j] == min(sizes[j], s*b) for all j."""
    D = len(sizes)
    b = B // D
    if cursors[0] < sizes[0]:
        if cursors[0] % b:
            raise ValueError("cursor of partition 0 is not at a step boundary")
        s = cursors[0] // b
    else:
        s = -(-sizes[0] // b)
    for j in range(D):
        if cursors[j] != min(sizes[j], s * b):
            raise ValueError(f"cursor of partition {j} is inconsistent with step {s}")
    return s


def repartition(parts: list, cursors: list, B: int, D_dst: int):
    """(new partitions, new cursors) for D_dst replicas, same global batch B."""
    s = steps_done([len(p) for p in parts], list(cursors), B)
    G = global_order(parts, B)
    new_parts = partition(G, B, D_dst)
    b2 = B // D_dst
    new_cursors = [int(min(len(p), s * b2)) for p in new_parts]
    return new_parts, new_cursors
