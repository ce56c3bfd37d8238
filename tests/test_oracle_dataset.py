"""Pins of the dataset-state oracle: a step-by-step simulation of data-parallel
consumption (independent of the oracle's index formula) and the consistency
requirements the paper states (sections 1 and 2.2: every sample exactly once per
epoch, consumption order unchanged by a re-partitioning, constant global batch)."""
import os

import numpy as np
import pytest

import synth
from oracle import dataset as ods


def simulate(parts, B, start_cursors=None, steps=None):
    """Run the data-parallel loop: at each step replica j takes its next B/D entries.
    Returns the samples in the order the job as a whole consumes them (step-major,
    replica-minor) and the cursors afterwards."""
    D = len(parts)
    b = B // D
    cur = list(start_cursors) if start_cursors is not None else [0] * D
    out = []
    k = 0
    while (steps is None or k < steps) and any(cur[j] < len(parts[j]) for j in range(D)):
        for j in range(D):
            take = parts[j][cur[j]:cur[j] + b]
            out.extend(int(x) for x in take)
            cur[j] += len(take)
        k += 1
    return out, cur


@pytest.mark.parametrize("n,B,D", [(48, 12, 3), (50, 12, 3), (53, 12, 4), (7, 12, 6), (100, 24, 6), (101, 24, 4), (0, 12, 2)])
def test_partition_consumes_global_order(n, B, D):
    G = synth.epoch_order(n, 7) if n else np.zeros(0, dtype=np.uint64)
    parts = ods.partition(G, B, D)
    order, cur = simulate(parts, B)
    assert order == [int(x) for x in G]                       # exactly once, in the global order
    assert cur == [len(p) for p in parts]
    assert np.array_equal(ods.global_order(parts, B), G)


@pytest.mark.parametrize("n,B,D,D2,s", [(100, 24, 6, 4, 2), (101, 24, 4, 6, 3), (53, 12, 2, 3, 0), (53, 12, 3, 1, 4),
                                        (53, 12, 3, 4, 5), (96, 24, 6, 4, 4), (200, 24, 6, 4, 9)])
def test_repartition_continues_the_same_order(n, B, D, D2, s):
    G = synth.epoch_order(n, 3)
    parts = ods.partition(G, B, D)
    before, cur = simulate(parts, B, steps=s)
    assert cur == ods.cursors_after(n, B, D, s)
    new_parts, new_cur = ods.repartition(parts, cur, B, D2)
    after, _ = simulate(new_parts, B, start_cursors=new_cur)
    assert before + after == [int(x) for x in G]              # nothing lost, repeated or reordered
    consumed_new = sorted(int(x) for j in range(D2) for x in new_parts[j][:new_cur[j]])
    assert consumed_new == sorted(before)                     # consumed set carried over
    assert sorted(int(x) for p in new_parts for x in p) == list(range(n))


def test_same_degree_is_identity_and_round_trip():
    G = synth.epoch_order(1000, 9)
    parts = ods.partition(G, 48, 6)
    cur = ods.cursors_after(1000, 48, 6, 11)
    same, cur_same = ods.repartition(parts, cur, 48, 6)
    assert all(np.array_equal(a, b) for a, b in zip(parts, same)) and cur_same == cur
    four, cur4 = ods.repartition(parts, cur, 48, 4)
    back, cur_back = ods.repartition(four, cur4, 48, 6)
    assert all(np.array_equal(a, b) for a, b in zip(parts, back)) and cur_back == cur


def test_ragged_tail_of_the_benchmark_shape():
    """B = 768, D 6 -> 4 with a tail of 256 samples: the tail lands on replicas 0 and 1 in
    both layouts, as 128 + 128 and as 192 + 64."""
    n, B = 768 * 5 + 256, 768
    G = synth.epoch_order(n, 6)
    p6, p4 = ods.partition(G, B, 6), ods.partition(G, B, 4)
    assert [len(p) for p in p6] == [5 * 128 + 128, 5 * 128 + 128, 640, 640, 640, 640]
    assert [len(p) for p in p4] == [5 * 192 + 192, 5 * 192 + 64, 960, 960]


def test_inconsistent_cursors_are_rejected():
    G = synth.epoch_order(100, 1)
    parts = ods.partition(G, 24, 4)
    with pytest.raises(ValueError):
        ods.repartition(parts, [6, 6, 6, 5], 24, 2)
    with pytest.raises(ValueError):
        ods.repartition(parts, [7, 7, 7, 7], 24, 2)
    with pytest.raises(ValueError):
        ods.partition(G, 25, 4)


def test_hand_worked_two_to_four_replicas_golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "dataset_d2_to_d4.txt")
    rows = [[int(x) for x in line.split()] for line in open(path) if line.strip() and not line.startswith("#")]
    two, four, cur2, cur4 = rows[0:2], rows[2:6], rows[6], rows[7]
    G = np.arange(11, dtype=np.uint64)
    assert [list(map(int, p)) for p in ods.partition(G, 4, 2)] == two
    assert [list(map(int, p)) for p in ods.partition(G, 4, 4)] == four
    assert ods.cursors_after(11, 4, 2, 1) == cur2
    parts, cur = ods.repartition([np.array(p, dtype=np.uint64) for p in two], cur2, 4, 4)
    assert [list(map(int, p)) for p in parts] == four and cur == cur4


def test_pair_entries_move_like_their_ids():
    """(offset, length) entries (section 5.2): a sample's two words travel together - column 0 of the
    re-partitioned pairs is the re-partitioned id array, column 1 the same function of it as before."""
    n, B = 1000, 48
    G = synth.epoch_order(n, 4)
    pairs = np.stack([G, G * np.uint64(7) + np.uint64(1)], axis=1)
    cur = ods.cursors_after(n, B, 6, 5)
    ids4, cur_ids = ods.repartition(ods.partition(G, B, 6), cur, B, 4)
    pairs4, cur_pairs = ods.repartition(ods.partition(pairs, B, 6), cur, B, 4)
    assert cur_ids == cur_pairs
    for a, b in zip(ids4, pairs4):
        assert np.array_equal(b[:, 0], a) and np.array_equal(b[:, 1], a * np.uint64(7) + np.uint64(1))


def cursors_by_counting(sizes, cursors, B, D2):
    """New cursors derived without any notion of a step: the global positions the old replicas have consumed (the
    first cursors[j] positions that belong to replica j), counted per replica of the new degree."""
    n, D = sum(sizes), len(sizes)
    b, b2 = B // D, B // D2
    consumed = []
    for j in range(D):
        mine = [p for p in range(n) if (p % B) // b == j]
        assert len(mine) == sizes[j]
        consumed += mine[:cursors[j]]
    return [sum(1 for p in consumed if (p % B) // b2 == j2) for j2 in range(D2)]


@pytest.mark.parametrize("n,B,D,D2", [(100, 24, 6, 4), (101, 24, 4, 6), (53, 12, 2, 3), (53, 12, 3, 4), (7, 12, 6, 4),
                                      (5, 8, 4, 2), (13, 8, 4, 2), (10, 8, 2, 4), (29, 12, 3, 6), (96, 24, 6, 4)])
def test_new_cursors_equal_a_count_of_consumed_positions(n, B, D, D2):
    G = synth.epoch_order(n, 11)
    parts = ods.partition(G, B, D)
    for s in range(-(-n // B) + 2):          # every step count up to and past the end of the epoch
        cur = ods.cursors_after(n, B, D, s)
        _, new_cur = ods.repartition(parts, cur, B, D2)
        assert new_cur == cursors_by_counting([len(p) for p in parts], cur, B, D2), s


def _ragged_cases():
    path = os.path.join(os.path.dirname(__file__), "golden", "dataset_ragged_tails.txt")
    lines = [l.split("#")[0].strip() for l in open(path)]
    lines = [l for l in lines if l]
    cases, i = [], 0
    while i < len(lines):
        n, D, D2 = (int(x) for x in lines[i].split())
        rows = [[] if l == "-" else [int(x) for x in l.split()] for l in lines[i + 1:i + 1 + D + D2]]
        i += 1 + D + D2
        steps = []
        while i < len(lines) and ":" in lines[i]:
            s, a, b = lines[i].split(":")
            steps.append((int(s), [int(x) for x in a.split()], [int(x) for x in b.split()]))
            i += 1
        cases.append((n, D, D2, rows[:D], rows[D:], steps))
    return cases


def test_hand_worked_ragged_tails_golden():
    """Global batch 8: a tail shorter than a local batch, a tail spanning several partitions, fewer samples than a batch."""
    cases = _ragged_cases()
    assert [c[0] for c in cases] == [10, 13, 5]
    for n, D, D2, old, new, steps in cases:
        G = np.arange(n, dtype=np.uint64)
        assert [list(map(int, p)) for p in ods.partition(G, 8, D)] == old
        assert [list(map(int, p)) for p in ods.partition(G, 8, D2)] == new
        for s, cur, cur2 in steps:
            assert ods.cursors_after(n, 8, D, s) == cur and ods.cursors_after(n, 8, D2, s) == cur2
            parts, got = ods.repartition([np.array(p, dtype=np.uint64) for p in old], cur, 8, D2)
            assert [list(map(int, p)) for p in parts] == new and got == cur2, (n, s)
            assert cursors_by_counting([len(p) for p in old], cur, 8, D2) == cur2


def test_pins_catch_a_floor_instead_of_ceiling_at_the_epoch_end(monkeypatch):
    """Planted mistake: taking floor(size / b) whole steps when partition 0 is exhausted loses the ragged last step."""
    real = ods.steps_done

    def wrong(sizes, cursors, B):
        b = B // len(sizes)
        if cursors[0] >= sizes[0]:
            return sizes[0] // b
        return real(sizes, cursors, B)
    monkeypatch.setattr(ods, "steps_done", wrong)
    with pytest.raises(AssertionError):
        test_hand_worked_ragged_tails_golden()
    monkeypatch.setattr(ods, "steps_done", real)
    test_hand_worked_ragged_tails_golden()
