"""Oracles for the multi-iteration decode loop around the attention kernel.

TEST INFRASTRUCTURE ONLY: plain NumPy / Python; shares no code with the
library.

kv_append -- paper Section 2.1: once a token is generated its key and value
are appended to the end of the request's KVCache and take part in every later
iteration.  In the paged layout, the new token of request b goes to position
kv_lens[b]: row kv_lens[b] % bs of physical block
block_table[b, kv_lens[b] // bs]; the length then grows by one.

BatchScheduler -- paper Section 3.4, Algorithm 2 (batch-level scheduling),
run after every decode iteration:
    release the HBM of completed requests and drop them from the running batch;
    if the next iteration does not fit in HBM       -> case 3: evict a victim to
        the candidate-requests buffer (the longest request; while two batches
        coexist, the longest request of the OLD batch);
    else if the candidate-requests buffer is not empty -> case 1: admit from it;
    else if the candidate-batch buffer is not empty    -> case 2: admit from it
        (the running batch then holds two original batches: a batch switch).
Readings where the listing leaves things open (listed in the design notes):
  * a request holds ceil(kv_len / bs) blocks; the next iteration needs one
    fresh block for every running request whose kv_len is a multiple of bs;
    "sufficient HBM" = that many blocks are free;
  * eviction repeats until the next iteration fits (the listing shows one
    victim; the prose speaks of "some requests");
  * admission takes requests in buffer order while the running batch is below
    `max_batch` and the request's blocks plus next-iteration growth still fit;
    it stops at the first request that does not fit;
  * "batch switching" = the running batch holds requests of more than one
    original batch; the old batch is the one with the smallest batch number;
  * longest = largest kv_len, earliest position in the running batch on ties;
  * an evicted request keeps its original batch number and joins the tail of
    the candidate-requests buffer.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np


def kv_append(k_blocks, v_blocks, block_table, kv_lens, k_new, v_new):
    """In place: write k_new[b], v_new[b] ([H_kv][D]) at position kv_lens[b]
    of every request and increment kv_lens[b]."""
    bs = k_blocks.shape[2]
    for b in range(len(kv_lens)):
        pos = int(kv_lens[b])
        blk = int(block_table[b, pos // bs])
        k_blocks[blk, :, pos % bs, :] = k_new[b]
        v_blocks[blk, :, pos % bs, :] = v_new[b]
        kv_lens[b] = pos + 1


@dataclass
class SchedRequest:
    id: int
    kv_len: int
    remaining: int     # tokens still to generate
    origin: int        # number of the batch the generator put it in


class BatchScheduler:
    def __init__(self, total_blocks: int, block_size: int = 16, max_batch: int = 64):
        self.bs = block_size
        self.free = int(total_blocks)
        self.total = int(total_blocks)
        self.max_batch = max_batch
        self.running: List[SchedRequest] = []
        self.r_cand: List[SchedRequest] = []
        self.b_cand: List[SchedRequest] = []

    def blocks(self, r: SchedRequest) -> int:
        return (r.kv_len + self.bs - 1) // self.bs

    def push_candidate_batch(self, origin, ids, kv_lens, remaining):
        for i, l, m in zip(ids, kv_lens, remaining):
            self.b_cand.append(SchedRequest(int(i), int(l), int(m), int(origin)))

    def push_candidate_request(self, origin, rid, kv_len, remaining):
        self.r_cand.append(SchedRequest(int(rid), int(kv_len), int(remaining), int(origin)))

    def _growth(self) -> int:
        return sum(1 for r in self.running if r.kv_len % self.bs == 0)

    def step(self, advance: bool = True):
        """One pass of Algorithm 2.  With advance=True every running request
        has just produced a token (kv_len + 1, remaining - 1).  Returns
        (completed ids, evicted ids, admitted ids, case) with case 0 (nothing
        to do), 1, 2 or 3."""
        if advance:
            for r in self.running:
                before = self.blocks(r)
                r.kv_len += 1
                r.remaining -= 1
                self.free -= self.blocks(r) - before
        completed = [r for r in self.running if r.remaining <= 0]
        for r in completed:
            self.free += self.blocks(r)
        self.running = [r for r in self.running if r.remaining > 0]
        evicted, admitted, case = [], [], 0
        if self._growth() > self.free:                                   # case 3
            case = 3
            while self.running and self._growth() > self.free:
                origins = {r.origin for r in self.running}
                pool = self.running
                if len(origins) > 1:
                    old = min(origins)
                    pool = [r for r in self.running if r.origin == old]
                victim = pool[0]
                for r in pool:
                    if r.kv_len > victim.kv_len:
                        victim = r
                self.running.remove(victim)
                self.free += self.blocks(victim)
                self.r_cand.append(victim)
                evicted.append(victim.id)
        else:
            source = None
            if self.r_cand:
                source, case = self.r_cand, 1
            elif self.b_cand:
                source, case = self.b_cand, 2
            if source is not None:
                while source and len(self.running) < self.max_batch:
                    r = source[0]
                    need = self.blocks(r) + self._growth() + (1 if r.kv_len % self.bs == 0 else 0)
                    if need > self.free:
                        break
                    source.pop(0)
                    self.free -= self.blocks(r)
                    self.running.append(r)
                    admitted.append(r.id)
                if not admitted:
                    case = 0
        return [r.id for r in completed], evicted, admitted, case
