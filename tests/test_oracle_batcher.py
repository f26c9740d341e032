"""Pins for the batcher oracle: a hand-worked case, the closed-form optimum,
and brute force over every partition on tiny inputs."""
import itertools
import json
import os

import numpy as np
import pytest

from oracle import batcher as ob

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_case():
    g = json.load(open(os.path.join(GOLD, "batcher_small.json")))
    order, offs = ob.aligned_batch(g["kv_lens"], g["batch_size"])
    assert order == g["order"]
    assert offs == g["batch_offsets"]
    assert ob.sum_of_batch_max(g["kv_lens"], order, offs) == g["sum_of_batch_max"]
    n = len(g["kv_lens"])
    arrival = list(range(n))
    assert ob.sum_of_batch_max(g["kv_lens"], arrival, [0, 3, 6, 7]) == g["arrival_order_sum_of_batch_max"]


def _all_partitions_min(lens, B):
    """Minimum of sum-of-batch-max over EVERY assignment of requests to at
    most ceil(n/B) groups of size <= B (exhaustive)."""
    n = len(lens)
    k = (n + B - 1) // B
    best = None
    for assign in itertools.product(range(k), repeat=n):
        # canonical labelling only (first occurrence order) to cut symmetry
        seen = -1
        ok = True
        for a in assign:
            if a > seen + 1:
                ok = False
                break
            seen = max(seen, a)
        if not ok:
            continue
        sizes = [0] * k
        mx = [0] * k
        for i, a in enumerate(assign):
            sizes[a] += 1
            mx[a] = max(mx[a], lens[i])
        if max(sizes) > B:
            continue
        tot = sum(mx)
        best = tot if best is None else min(best, tot)
    return best


@pytest.mark.parametrize("n,B", [(1, 2), (4, 2), (5, 2), (6, 3), (7, 3), (8, 4), (9, 4), (7, 2), (9, 3)])
def test_brute_force_optimality(n, B):
    rng = np.random.default_rng(100 * n + B)
    for trial in range(4):
        if trial == 0:
            lens = rng.integers(1, 50, n).tolist()
        elif trial == 1:
            lens = rng.integers(1, 4, n).tolist()          # heavy ties
        elif trial == 2:
            lens = [7] * n                                   # all equal
        else:
            lens = sorted(rng.integers(1, 1000, n).tolist())  # adversarial for ascending chunking
        order, offs = ob.aligned_batch(lens, B)
        got = ob.sum_of_batch_max(lens, order, offs)
        assert got == _all_partitions_min(lens, B), (lens, B)


def test_closed_form_and_structure():
    rng = np.random.default_rng(5)
    for _ in range(200):
        n = int(rng.integers(0, 70))
        B = int(rng.integers(1, 12))
        lens = rng.integers(1, 40, n).tolist()
        order, offs = ob.aligned_batch(lens, B)
        nb = (n + B - 1) // B
        assert sorted(order) == list(range(n))
        assert offs[0] == 0 and offs[-1] == n and len(offs) == nb + 1
        sizes = [b - a for a, b in zip(offs[:-1], offs[1:])]
        assert all(s == B for s in sizes[:-1]) and (not sizes or 1 <= sizes[-1] <= B)
        srt = [lens[i] for i in order]
        assert all(a >= b for a, b in zip(srt[:-1], srt[1:]))
        for a, b in zip(order[:-1], order[1:]):
            if lens[a] == lens[b]:
                assert a < b                        # ties keep index order
        d = sorted(lens, reverse=True)
        assert ob.sum_of_batch_max(lens, order, offs) == sum(d[k * B] for k in range(nb))


def test_short_batch_holds_the_shortest_requests():
    lens = [10, 20, 30, 40, 50]
    order, offs = ob.aligned_batch(lens, 2)
    assert order == [4, 3, 2, 1, 0] and offs == [0, 2, 4, 5]
    # putting the remainder at the long end costs more
    assert ob.sum_of_batch_max(lens, order, offs) == 90
    assert ob.sum_of_batch_max(lens, [0, 1, 2, 3, 4], [0, 2, 4, 5]) == 110


def test_edge_cases():
    assert ob.aligned_batch([], 4) == ([], [0])
    assert ob.aligned_batch([5], 4) == ([0], [0, 1])
    assert ob.aligned_batch([5, 9, 1], 8) == ([1, 0, 2], [0, 3])
    with pytest.raises(ValueError):
        ob.aligned_batch([1, 2], 0)
