"""The C++ batch-level scheduler against its oracle: identical events and
state on the hand-worked traces and on random traces.  Host only."""
import json
import os

import numpy as np
import pytest

from oracle import decode_loop as od
from paper_2605_23389_amd import binding as als

GOLD = os.path.join(os.path.dirname(__file__), "golden", "scheduler_cases.json")


def test_hand_worked_traces_through_the_abi(lib):
    g = json.load(open(GOLD))
    for sc in g["scenarios"]:
        s = lib.Scheduler(sc["total_blocks"], 16, sc["max_batch"])
        for st in sc["steps"]:
            if "push_batch" in st:
                p = st["push_batch"]
                s.push_candidate_batch(p["origin"], p["ids"], p["kv_lens"], p["remaining"])
            if "push_request" in st:
                p = st["push_request"]
                s.push_candidate_request(p["origin"], p["id"], p["kv_len"], p["remaining"])
            for _ in range(st.get("repeat", 1)):
                done, ev, ad, case = s.step(st["advance"])
                assert [done, ev, ad, case] == st["expect"], (sc["name"], st)
                assert s.state()["free_blocks"] == st["free"]


def test_random_traces_match_oracle(lib):
    rng = np.random.default_rng(8)
    for trial in range(60):
        total = int(rng.integers(8, 300))
        mb = int(rng.integers(1, 24))
        s, o = lib.Scheduler(total, 16, mb), od.BatchScheduler(total, 16, mb)
        origin, next_id = 0, 0
        for it in range(200):
            if rng.random() < 0.3:
                n = int(rng.integers(1, 12))
                ids = np.arange(next_id, next_id + n)
                L = rng.integers(1, 16 * max(total // 3, 1), n)
                R = rng.integers(1, 50, n)
                s.push_candidate_batch(origin, ids, L, R)
                o.push_candidate_batch(origin, ids, L, R)
                origin += 1
                next_id += n
            if rng.random() < 0.1:
                L, R = int(rng.integers(1, 200)), int(rng.integers(1, 30))
                s.push_candidate_request(max(origin - 1, 0), next_id, L, R)
                o.push_candidate_request(max(origin - 1, 0), next_id, L, R)
                next_id += 1
            got = s.step(it > 0)
            want = o.step(it > 0)
            assert got == (want[0], want[1], want[2], want[3]), (trial, it)
            st = s.state()
            assert st["free_blocks"] == o.free and st["running"] == len(o.running)
            assert st["candidate_requests"] == len(o.r_cand) and st["candidate_batch"] == len(o.b_cand)
            ids, lens, org = s.running()
            assert ids.tolist() == [r.id for r in o.running]
            assert lens.tolist() == [r.kv_len for r in o.running]
            assert org.tolist() == [r.origin for r in o.running]


def test_scheduler_errors(lib):
    with pytest.raises(als.AlignedServeError):
        lib.Scheduler(0, 16, 4)
    s = lib.Scheduler(10, 16, 4)
    with pytest.raises(als.AlignedServeError):
        s.push_candidate_batch(0, [1], [0], [5])
    with pytest.raises(als.AlignedServeError):
        s.push_candidate_request(0, 1, 5, 0)
    assert s.step(False) == ([], [], [], 0)
