"""Pins for the quad-tree / Density First Search oracle (paper Section 3.3,
Algorithm 1): hand-worked scenarios, one per case, and invariants on random
inputs.

Derivations of the golden scenarios (tree [1,64], leaf width 4):
 * case1_whole_tree: the root holds 8 blocks <= 100 and 4 >= 3 requests.
 * case2_descend: root 17 blocks > 6 -> densest child [1,16] (3 requests,
   6 blocks <= 6, 3 >= 2) is the batch; then root 11 > 6 -> child [17,32]
   (2 requests beat 1), 6 blocks, 2 >= 2; then root 5 <= 6 but 1 < 2: case 3 at
   the root, which has no siblings -> the single request.
 * case3_right: root 13 > 10 -> child [17,32] (6 requests), 12 > 10 -> leaves
   hold 2,1,2,1 requests, tie -> leftmost leaf [17,20] = {0,1}, 3 blocks, 2 < 4:
   case 3 with B_left 7, K_left 2, no left sibling -> scan right siblings left
   to right: r2 (3) ok, r3 (5) ok, r4 (7) ok, r5 (9 > 7) stop -> [2,3,4] cut
   to K_left = 2 -> batch 0,1,2,3.  Then root 5 <= 10, 3 < 4 -> all three.
 * case3_left: root 14 > 10 -> child [17,32]; leaves hold 1,2,2,3 requests ->
   leaf [29,32] = {4,5,6}, 3 blocks, 3 < 4: B_left 7, K_left 1; left siblings
   scanned from the nearest, longest request first: r7 (2), r3 (5), r2 (6),
   r1 (7), r0 (11 > 7) stop -> [7,3,2,1] cut to 1 -> batch 4,5,6,7.  Then the
   root holds 9 <= 10 blocks and 4 >= 4 requests: case 1.
 * leaf_overflow: one leaf holds 9 blocks > 5: requests are taken in order
   while they fit (3, then 6 > 5); length 1000 is clamped to 64.
"""
import json
import os

import numpy as np
import pytest

from oracle import quadtree as oq

GOLD = os.path.join(os.path.dirname(__file__), "golden", "quadtree_cases.json")


def _run(sc, geom):
    t = oq.QuadTree(**geom)
    for rid, length, blocks in sc["requests"]:
        t.insert(rid, length, blocks)
    batches, cases = [], []
    while len(t):
        batches.append(t.next_batch(sc["b_max"], sc["k_min"]))
        cases.append(t.last_case)
    return batches, cases


def test_hand_worked_scenarios():
    g = json.load(open(GOLD))
    for sc in g["scenarios"]:
        batches, cases = _run(sc, g["geometry"])
        assert batches == sc["batches"], sc["name"]
        assert cases == sc["cases"], sc["name"]


def test_tree_geometry_and_counters():
    t = oq.QuadTree(65536, 16)
    depth, n = 0, t.root
    while not n.is_leaf():
        assert len(n.children) == 4
        widths = {c.hi - c.lo + 1 for c in n.children}
        assert len(widths) == 1 and n.children[0].lo == n.lo and n.children[3].hi == n.hi
        n, depth = n.children[2], depth + 1
    assert depth == 6 and n.hi - n.lo + 1 == 16
    t.insert(1, 70000, 5)      # clamped to 65536
    t.insert(2, 1, 2)
    t.insert(3, 16, 1)
    t.insert(4, 17, 1)
    assert t.request_counter(t.root) == 4 and t.block_counter(t.root) == 9
    assert [r.id for r in t.collect(t.root)] == [2, 3, 4, 1]
    assert t.request_counter(t.root.children[0]) == 3 and t.request_counter(t.root.children[3]) == 1
    with pytest.raises(ValueError):
        oq.QuadTree(100, 16)
    with pytest.raises(ValueError):
        t.insert(1, 5, 1)


def _subtree_ids(t, node):
    return {r.id for r in t.collect(node)}


def test_invariants_on_random_inputs():
    rng = np.random.default_rng(3)
    for trial in range(25):
        n = int(rng.integers(1, 80))
        lens = np.clip(np.rint(np.exp(rng.normal(np.log(300), 1.2, n))), 1, 5000).astype(int)
        blocks = (lens + 15) // 16
        b_max = int(rng.integers(int(blocks.max()), int(blocks.sum()) + 2))
        k_min = int(rng.integers(1, 12))
        t = oq.QuadTree(4096 * 4, 16)
        for i in range(n):
            t.insert(i, int(lens[i]), int(blocks[i]))
        seen = []
        while len(t):
            before = {nid: None for nid in _subtree_ids(t, t.root)}
            # remember sub-tree membership before the batch is removed
            ids = None
            snapshot = oq.QuadTree(4096 * 4, 16)
            for r in t.collect(t.root):
                snapshot.insert(r.id, r.length, r.blocks)
            ids = t.next_batch(b_max, k_min)
            assert ids and len(set(ids)) == len(ids) and set(ids) <= set(before)
            used = int(sum(blocks[i] for i in ids))
            assert used <= b_max or len(ids) == 1
            node = t.last_node
            # the same node in the snapshot
            sn = snapshot.root
            while (sn.lo, sn.hi) != (node.lo, node.hi):
                q = (sn.hi - sn.lo + 1) // 4
                sn = sn.children[(node.lo - sn.lo) // q]
            own = _subtree_ids(snapshot, sn)
            if t.last_case == 1:
                assert set(ids) == own and len(ids) >= k_min
            elif t.last_case == 3:
                assert own <= set(ids) and len(ids) <= max(k_min, len(own))
                extra = set(ids) - own
                if extra:
                    assert sn.parent is not None and extra <= _subtree_ids(snapshot, sn.parent)
                    left = set().union(*[_subtree_ids(snapshot, c) for c in sn.parent.children[:sn.slot]]) \
                        if sn.slot else set()
                    assert extra <= left if sn.slot else not (extra & own)
            else:
                assert sn.is_leaf() and set(ids) <= own
            seen.extend(ids)
        assert sorted(seen) == list(range(n))


def test_dfs_batches_wrapper_and_similarity():
    rng = np.random.default_rng(9)
    lens = np.clip(np.rint(np.exp(rng.normal(np.log(1024), 1.2, 250))), 64, 32768).astype(int)
    blocks = (lens + 15) // 16
    order, offs = oq.dfs_batches(lens, blocks, b_max=int(blocks.sum() * 0.1), k_min=36)
    assert sorted(order) == list(range(250)) and offs[0] == 0 and offs[-1] == 250
    # batches are tighter in length than arrival-order groups of the same sizes
    def spread(o):
        return sum(lens[o[a:b]].max() - lens[o[a:b]].min() for a, b in zip(offs[:-1], offs[1:]))
    assert spread(np.array(order)) < 0.5 * spread(np.arange(250))


def test_starving_subtree_is_served_first():
    t = oq.QuadTree(64, 4)
    for i in range(6):
        t.insert(i, 5 + (i % 3), 1, now=0.0)          # dense short requests
    t.insert(100, 60, 1, now=0.0)                      # a lonely long one
    # without the starvation rule the dense sub-tree wins (b_max forces a descent)
    t2 = oq.QuadTree(64, 4)
    for i in range(6):
        t2.insert(i, 5 + (i % 3), 1)
    t2.insert(100, 60, 1)
    assert 100 not in t2.next_batch(6, 2)
    # the dense leaves keep producing batches; the long request's sub-tree ages
    ids = t.next_batch(3, 2, now=1.0, starve_after=10.0)
    assert 100 not in ids
    ids = t.next_batch(3, 2, now=20.0, starve_after=10.0)
    assert 100 in ids
