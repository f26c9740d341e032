"""Pins for the decode-loop oracles: KV append (paper Section 2.1) and the
batch-level scheduling policy (Section 3.4, Algorithm 2).

Derivations of the scheduler goldens (block size 16):
 * eviction...: 5 blocks.  r1 (16 tokens, 1 block, needs a fresh block next
   iteration) and r2 (31 tokens, 2 blocks) are admitted: 1+1 <= 5, then
   2 + 1 (r1's growth) <= 4; free 2.  Iteration 1: r1 -> 17 (2 blocks, free 1),
   r2 -> 32: growth 1 <= 1.  Iteration 2: r2 -> 33 (3 blocks, free 0).  Thirteen
   quiet iterations bring r1 to 31, r2 to 46.  Next: r1 = 32 needs a block,
   none is free -> case 3: one batch only, the longest is r2 (47 tokens,
   3 blocks) -> evicted, free 3.  Next: r1 -> 33 (3 blocks, free 2); the
   candidate-requests buffer holds r2 (3 blocks > 2): nothing admitted.
 * batch switch: 8 blocks.  r1 (40 tokens, 3 blocks) runs alone (free 5); batch
   1 = r2 (15 tokens, 1 block), r3 (60 tokens, 4 blocks) is admitted (free 0):
   two original batches coexist.  Next iteration r2 reaches 16 and needs a
   block: case 3 while switching -> the longest request of the OLD batch, r1
   (42 tokens), goes, although r3 (61 tokens) is longer.
 * refill: 7 blocks, at most 3 running.  r10 (30 tokens, 2 tokens left), r11
   admitted (free 3).  A late request r12 of batch 0 sits in the candidate-
   requests buffer and batch 1 in the candidate-batch buffer: the requests
   buffer is served first (case 1), r12 (18 tokens, 2 blocks) fits (free 1) and
   fills the batch.  Next iteration r10 -> 32 with 0 left: it completes and its
   2 blocks are released (free 3); the same pass then continues as the listing
   does: HBM suffices, the requests buffer is empty, so case 2 admits r20 (31
   tokens, 2 blocks <= 3; free 1) and the batch is full again.  Next iteration
   r20 -> 32 needs a fresh block next time (1 <= 1 free); r21 cannot join a full
   batch: nothing happens.
"""
import json
import os

import numpy as np

from oracle import attention as oa
from oracle import decode_loop as od
from paper_2605_23389_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "scheduler_cases.json")


def test_kv_append_then_gather_is_concatenation():
    rng = np.random.default_rng(0)
    lens = np.array([15, 16, 31, 1], dtype=np.int32)
    pb = wl.make_paged_batch(lens + 3, 2, 2, 8, dtype="fp32", seed=1)   # room for 3 more tokens
    cur = lens.copy()
    before = [oa.gather_kv(pb.k_blocks, pb.block_table[b], cur[b], 1) for b in range(4)]
    added = []
    for step in range(3):
        k_new = rng.standard_normal((4, 2, 8)).astype(np.float32)
        v_new = rng.standard_normal((4, 2, 8)).astype(np.float32)
        od.kv_append(pb.k_blocks, pb.v_blocks, pb.block_table, cur, k_new, v_new)
        added.append((k_new, v_new))
    assert cur.tolist() == (lens + 3).tolist()
    for b in range(4):
        got_k = oa.gather_kv(pb.k_blocks, pb.block_table[b], cur[b], 1)
        want_k = np.concatenate([before[b]] + [a[0][b, 1][None] for a in added])
        assert np.array_equal(got_k, want_k)
        got_v = oa.gather_kv(pb.v_blocks, pb.block_table[b], cur[b], 0)
        assert np.array_equal(got_v[-3:], np.stack([a[1][b, 0] for a in added]))


def _play(sc):
    s = od.BatchScheduler(sc["total_blocks"], 16, sc["max_batch"])
    log = []
    for st in sc["steps"]:
        if "push_batch" in st:
            p = st["push_batch"]
            s.push_candidate_batch(p["origin"], p["ids"], p["kv_lens"], p["remaining"])
        if "push_request" in st:
            p = st["push_request"]
            s.push_candidate_request(p["origin"], p["id"], p["kv_len"], p["remaining"])
        for _ in range(st.get("repeat", 1)):
            out = s.step(st["advance"])
            log.append((list(map(list, out[:3])) + [out[3]], s.free))
            assert list(map(list, out[:3])) + [out[3]] == st["expect"], (sc["name"], st, out)
            assert s.free == st["free"], (sc["name"], st, s.free)
    return log


def test_hand_worked_scheduler_scenarios():
    g = json.load(open(GOLD))
    for sc in g["scenarios"]:
        _play(sc)


def test_scheduler_invariants_on_random_traces():
    rng = np.random.default_rng(4)
    for trial in range(40):
        total = int(rng.integers(8, 200))
        s = od.BatchScheduler(total, 16, int(rng.integers(1, 20)))
        origin, next_id, alive = 0, 0, {}
        for it in range(150):
            if not s.b_cand and rng.random() < 0.5:
                n = int(rng.integers(1, 10))
                ids = list(range(next_id, next_id + n))
                L = rng.integers(1, 16 * max(total // 4, 1), n)
                R = rng.integers(1, 40, n)
                s.push_candidate_batch(origin, ids, L, R)
                for i, l in zip(ids, L):
                    alive[i] = int(l)
                origin += 1
                next_id += n
            done, ev, ad, case = s.step(advance=it > 0)
            held = sum(s.blocks(r) for r in s.running)
            assert held + s.free == total and s.free >= 0
            assert len(s.running) <= s.max_batch
            assert sum(1 for r in s.running if r.kv_len % 16 == 0) <= s.free or not s.running
            if case == 3:
                assert ev and not ad
            if ev:
                assert case == 3 and [r.id for r in s.r_cand][-len(ev):] == ev
            if case == 1:
                assert ad
            ids_now = [r.id for r in s.running] + [r.id for r in s.r_cand] + [r.id for r in s.b_cand]
            assert len(ids_now) == len(set(ids_now))
            for d in done:
                alive.pop(d)
            assert set(ids_now) == set(alive)
