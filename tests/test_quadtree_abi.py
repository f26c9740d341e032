"""The C++ quad-tree / Density First Search generator against its oracle,
bit-exact (same batches, same order inside each batch, same case), on the
hand-worked scenarios, random inputs, interleaved inserts/removes and the
starvation rule.  Host only."""
import json
import os

import numpy as np
import pytest

from oracle import quadtree as oq
from paper_2605_23389_amd import binding as als
from paper_2605_23389_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "quadtree_cases.json")


def test_hand_worked_scenarios_through_the_abi(lib):
    g = json.load(open(GOLD))
    for sc in g["scenarios"]:
        t = lib.QuadTree(**g["geometry"])
        for rid, length, blocks in sc["requests"]:
            t.insert(rid, length, blocks)
        got, cases = [], []
        while len(t):
            ids, case = t.next_batch(sc["b_max"], sc["k_min"])
            got.append(ids)
            cases.append(case)
        assert got == sc["batches"] and cases == sc["cases"], sc["name"]
        assert t.next_batch(sc["b_max"], sc["k_min"]) == ([], 0)


def test_random_inputs_match_oracle(lib):
    rng = np.random.default_rng(11)
    for trial in range(60):
        n = int(rng.integers(1, 120))
        geom = [(64, 4), (4096, 16), (1024, 1), (64, 4), (16384, 1024), (4096, 16)][trial % 6]
        if trial in (7, 31):
            geom = (65536, 16)                                # the paper's range (slow in the oracle)
        hi = geom[0] * (2 if trial % 7 == 0 else 1)          # sometimes beyond the clamp
        lens = np.clip(np.rint(np.exp(rng.normal(np.log(max(hi / 30, 2)), 1.3, n))), 1, hi).astype(np.int32)
        blocks = ((lens + 15) // 16).astype(np.int32)
        if trial % 3 == 0:
            blocks = rng.integers(1, 9, n).astype(np.int32)
        b_max = int(rng.integers(1, int(blocks.sum()) + 2))
        k_min = int(rng.integers(1, 40))
        o_order, o_offs = oq.dfs_batches(lens, blocks, b_max, k_min, *geom)
        order, offs = lib.dfs_batches(lens, blocks, b_max, k_min, *geom)
        assert order.tolist() == o_order and offs.tolist() == o_offs, (trial, geom, b_max, k_min)


def test_interleaved_updates_and_starvation_match_oracle(lib):
    rng = np.random.default_rng(5)
    for trial in range(30):
        geom = (4096, 16)
        t, o = lib.QuadTree(*geom), oq.QuadTree(*geom)
        next_id, now, live = 0, 0.0, []
        for step in range(60):
            now += float(rng.integers(1, 5))
            op = rng.integers(0, 4)
            if op <= 1 or not live:
                for _ in range(int(rng.integers(1, 12))):
                    L = int(np.clip(np.rint(np.exp(rng.normal(5.5, 1.2))), 1, 5000))
                    b = (min(L, 4096) + 15) // 16
                    t.insert(next_id, L, b, now)
                    o.insert(next_id, L, b, now)
                    live.append(next_id)
                    next_id += 1
            elif op == 2:
                rid = live.pop(int(rng.integers(0, len(live))))
                t.remove(rid)
                o.remove(rid)
            else:
                b_max, k_min = int(rng.integers(8, 200)), int(rng.integers(1, 10))
                starve = [None, 6.0, 15.0][int(rng.integers(0, 3))]
                ids, case = t.next_batch(b_max, k_min, now, starve)
                o_ids = o.next_batch(b_max, k_min, now, starve)
                assert ids == o_ids and case == o.last_case
                live = [x for x in live if x not in set(ids)]
            assert t.size() == (o.request_counter(o.root), o.block_counter(o.root))


def test_errors(lib):
    with pytest.raises(als.AlignedServeError):
        lib.QuadTree(100, 16)
    t = lib.QuadTree(64, 4)
    t.insert(1, 5, 1)
    for bad in ((1, 6, 1), (2, 0, 1), (3, 5, 0)):
        with pytest.raises(als.AlignedServeError) as e:
            t.insert(*bad)
        assert e.value.status == als.AS_EINVAL
    with pytest.raises(als.AlignedServeError):
        t.remove(99)
    with pytest.raises(als.AlignedServeError):
        t.next_batch(0, 1)
    assert t.size() == (1, 1)


def test_generator_on_the_benchmark_lengths(lib):
    """configs[2] lengths with the paper's parameters (K_min = 36; B_max = 40 % of
    a pool sized for a tenth of the in-flight blocks): every batch respects the
    budget and the batches are length-aligned (sum of batch maxima far below the
    random grouping's)."""
    from oracle import batcher as ob
    lens = wl.config_lengths(2)
    blocks = ((lens + 15) // 16).astype(np.int32)
    b_max = int(0.4 * blocks.sum() / 10)
    order, offs = lib.dfs_batches(lens, blocks, b_max, 36)
    assert sorted(order.tolist()) == list(range(len(lens)))
    for a, b in zip(offs[:-1], offs[1:]):
        assert blocks[order[a:b]].sum() <= b_max or b - a == 1
    # the oracle is quadratic: cross-check on the first 250 requests only
    sub_b = int(0.4 * blocks[:250].sum() / 10)
    o_order, o_offs = oq.dfs_batches(lens[:250], blocks[:250], sub_b, 36)
    s_order, s_offs = lib.dfs_batches(lens[:250], blocks[:250], sub_b, 36)
    assert s_order.tolist() == o_order and s_offs.tolist() == o_offs
    # length-aligned: the spread of lengths inside a batch is far below that of
    # a random grouping with the same batch sizes
    r_order, _ = wl.random_grouping(len(lens), 64, seed=0)

    def spread(o):
        return sum(int(lens[o[a:b]].max()) - int(lens[o[a:b]].min()) for a, b in zip(offs[:-1], offs[1:]))
    assert spread(order) < 0.25 * spread(r_order)
