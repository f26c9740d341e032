"""Multi-iteration decode simulation that drives the real library calls.

Plumbing only: it owns the HBM block free-list, the pinned host KV pool and
the per-iteration batch tensors, and calls the library for every step of the
path -- batch generation (as_qtree_* / arrival order), scheduling
(as_sched_step, paper Algorithm 2), KV migration (as_stage_kv /
as_unstage_kv on the as_pipeline_* side stream), KV append (as_kv_append) and
attention (as_decode_attention).  Prompts, model weights and sampled tokens do
not exist here: prefix lengths and output lengths are synthetic, queries and
new K/V rows are random.

One GPU stands in for the paper's pair of devices (Section 3.2, Fig. 4): the
decoding instance's HBM is a budget of `hbm_blocks` blocks, which is what the
scheduler manages; the Candidate Batch Buffer and the Candidate Requests
Buffer, which the paper keeps in a second GPU's memory, are a second budget of
`cand_blocks` blocks of the same physical pool.  With `prefetch` on, the next
generated batch (and requests waiting in the candidate-requests buffer) are
staged host -> HBM on the side stream while the running batch decodes
(Fig. 4 step 4, Section 4.4); when Algorithm 2 admits such a request its
blocks only change owner -- an edit of the block table, no copy on the
iteration's critical path.  With `prefetch` off a request is staged at the
moment it is admitted and the iteration waits for the copy: the bubble the
paper measures as the time to schedule an iteration (Section 4.3).
Evicted requests (Algorithm 2, case 3) leave through as_unstage_kv behind an
event; their blocks return to the free list when the copy has finished.

Per iteration, in the order of Section 2.2: the new token's k, v are appended
to the cache first (Eq. 1), then its query attends over all kv_len + 1 tokens
(Eq. 2).

`dry=True` runs the same logic without a GPU (data movement is recorded and
checked, not executed): the host-side bookkeeping can be tested anywhere.
"""
from __future__ import annotations

import time
from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import numpy as np

from . import binding as als

BS = 16  # tokens per KV block


@dataclass
class SimConfig:
    num_q_heads: int = 32
    num_kv_heads: int = 32
    head_dim: int = 128
    max_batch: int = 64
    hbm_blocks: int = 16384          # decode instance's block budget (what Algorithm 2 manages)
    cand_blocks: int = 0             # candidate-buffer budget; 0 => b_max_frac * hbm_blocks + 2 * longest request
    policy: str = "aligned"          # "aligned" (quad-tree DFS) or "fcfs" (arrival order)
    k_min: int = 36                  # paper Section 4.1
    b_max_frac: float = 0.4          # paper Section 4.1: 40 % of the GPU blocks
    starve_after: float = -1.0       # paper Section 3.5: a sub-tree that has waited longer than this many decode
                                     # iterations is served first (negative: off)
    prefetch: bool = True            # stage candidates ahead of admission (off: stage when admitted)
    prefetch_group_blocks: int = 256 # blocks per prefetch copy group (a request is never cut)
    prefetch_groups_in_flight: int = 2   # prefetch pauses while this many copy groups are unfinished
    stage_policy: str = "auto"       # how as_stage_kv moves blocks: "auto", "dma" or "kernel" (as_stage_set_policy)
    host_arena_blocks: int = 0       # 0 => one unique host block per logical block (verification runs)
    seed: int = 0
    verify_every: int = 0            # >0: compare device KV with a host mirror every n-th iteration
    evict_slots: int = 0             # host slots for evicted requests (0 => 2 * max_batch)
    dry: bool = False                # no GPU: bookkeeping only


# ---------------------------------------------------------------------------
# back ends: everything that touches the GPU sits behind this small interface
# ---------------------------------------------------------------------------
class _DryEvent:
    """Completes after `polls` queries (so that deferred frees are exercised)."""

    def __init__(self, polls: int):
        self.left = polls

    def query(self) -> bool:
        self.left -= 1
        return self.left < 0

    def synchronize(self):
        self.left = -1


class _DryBackend:
    """Records data movement instead of doing it."""

    def __init__(self, sim: "DecodeSim"):
        self.sim = sim
        self.moves: List[Tuple] = []
        self.tick = 0
        self.acquired: List[int] = []

    def stage(self, arena, src, dst):
        assert len(src) == len(dst)
        self.moves.append(("stage", arena, len(dst)))

    def unstage_behind_event(self, dst, src, nbytes):
        assert len(src) == len(dst)
        self.moves.append(("unstage", len(src)))
        return _DryEvent(polls=2)

    def outstanding(self) -> int:
        return 0

    def begin_group(self) -> int:
        self.tick += 1
        return self.tick

    def end_group(self, tick, nbytes, critical):
        pass

    def acquire(self, tick) -> bool:
        self.acquired.append(tick)
        return True

    def make_mirror(self, rid, start, nb, L):
        pass

    def iterate(self, rows, lens, it):
        return None

    def finish(self, stats):
        pass


class _GpuBackend:
    def __init__(self, sim: "DecodeSim"):
        import torch
        self.torch = torch
        self.sim = sim
        cfg = sim.cfg
        Hq, Hkv, D = cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim
        dev = "cuda"
        self.dev_k = torch.zeros((sim.pool_blocks, Hkv, BS, D), dtype=torch.bfloat16, device=dev)
        self.dev_v = torch.zeros_like(self.dev_k)
        g = torch.Generator().manual_seed(cfg.seed)
        self.host_k = torch.empty((sim.arena, Hkv, BS, D), dtype=torch.bfloat16, pin_memory=True)
        self.host_v = torch.empty_like(self.host_k, pin_memory=True)
        chunk = torch.randn((min(sim.arena, 256), Hkv, BS, D), generator=g).to(torch.bfloat16)
        for t in (self.host_k, self.host_v):
            for i in range(0, sim.arena, chunk.shape[0]):
                m = min(chunk.shape[0], sim.arena - i)
                t[i:i + m].copy_(chunk[:m] if not cfg.verify_every else
                                 torch.randn((m, Hkv, BS, D), generator=g).to(torch.bfloat16))
        self.evict_k = torch.empty((sim.evict_slots * sim.MB, Hkv, BS, D), dtype=torch.bfloat16, pin_memory=True)
        self.evict_v = torch.empty_like(self.evict_k, pin_memory=True)
        als.stage_set_policy({"auto": als.STAGE_AUTO, "dma": als.STAGE_DMA, "kernel": als.STAGE_KERNEL}[cfg.stage_policy])
        self.pipe = als.Pipeline(self.RING)
        self.side = torch.cuda.ExternalStream(self.pipe.stream)
        self.compute = torch.cuda.current_stream()
        self.gen = torch.Generator(device=dev).manual_seed(cfg.seed + 1)
        self.q_all = torch.empty((cfg.max_batch, Hq, D), dtype=torch.bfloat16, device=dev).normal_(generator=self.gen)
        self.out_all = torch.empty_like(self.q_all)
        self.knew = torch.empty((cfg.max_batch, Hkv, D), dtype=torch.bfloat16, device=dev)
        self.vnew = torch.empty_like(self.knew)
        self.bt_dev = torch.zeros((cfg.max_batch, sim.MB), dtype=torch.int32, device=dev)
        self.dl_dev = torch.zeros((cfg.max_batch,), dtype=torch.int32, device=dev)
        self.bt_pin = torch.zeros((cfg.max_batch, sim.MB), dtype=torch.int32, pin_memory=True)
        self.dl_pin = torch.zeros((cfg.max_batch,), dtype=torch.int32, pin_memory=True)
        self.ws = None
        self.ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(2)]
        self.copy_events: List[Tuple] = []     # (start, stop, bytes, kind)
        self.mirror: Dict[int, list] = {}
        self.tick = 0
        self.inflight: List[int] = []
        self.done_upto = 0
        self.block_bytes = sim.block_bytes

    # ---- data movement (all on the pipeline's side stream)
    def stage(self, arena, src, dst):
        hk, hv = (self.host_k, self.host_v) if arena == "host" else (self.evict_k, self.evict_v)
        als.stage_kv(hk, hv, src, self.dev_k, self.dev_v, dst, self.block_bytes, stream=self.pipe.stream)

    # Copy groups take the pipeline's 8 "ready" events in turn.  A slot is taken again only when
    # its previous group is known to have finished (at most RING - 1 groups are in flight), so
    # the event of a group that is still in flight always belongs to that group.
    RING = 8

    def outstanding(self) -> int:
        """Copy groups not yet known to have finished (polls the pipeline; the side stream is FIFO)."""
        while self.inflight and self.pipe.query(self.inflight[0] % self.RING):
            self.done_upto = self.inflight.pop(0)
        return len(self.inflight)

    def begin_group(self) -> int:
        while self.outstanding() >= self.RING - 1:
            self.side.synchronize()
        self.tick += 1
        self.pipe.begin_stage(self.tick % self.RING)
        e = self.torch.cuda.Event(enable_timing=True)
        e.record(self.side)
        self._group_start = e
        return self.tick

    def end_group(self, tick, nbytes, critical):
        e = self.torch.cuda.Event(enable_timing=True)
        e.record(self.side)
        self.copy_events.append((self._group_start, e, nbytes, "h2d_critical" if critical else "h2d_prefetch"))
        self.pipe.end_stage(tick % self.RING)
        self.inflight.append(tick)

    def acquire(self, tick) -> bool:
        """The compute stream waits for copy group `tick` -- unless it is known to have finished
        (returns True then: the request was resident)."""
        self.outstanding()
        if tick > self.done_upto:
            self.pipe.acquire(tick % self.RING, stream=self.compute)
            return False
        return True

    def unstage_behind_event(self, dst, src, nbytes):
        """Eviction copy on the side stream; returns the event that marks its end."""
        # the running batch's last attention has finished with the blocks (the loop synchronises
        # every iteration); the side stream still waits for the compute stream for good measure
        self.side.wait_stream(self.compute)
        e0 = self.torch.cuda.Event(enable_timing=True)
        e1 = self.torch.cuda.Event(enable_timing=True)
        e0.record(self.side)
        als.unstage_kv(self.evict_k, self.evict_v, dst, self.dev_k, self.dev_v, src, self.block_bytes,
                       stream=self.pipe.stream)
        e1.record(self.side)
        self.copy_events.append((e0, e1, nbytes, "d2h"))
        return e1

    def make_mirror(self, rid, start, nb, L):
        if not self.sim.cfg.verify_every:
            return
        torch = self.torch
        k = self.host_k[start:start + nb].view(torch.int16).numpy().copy()
        v = self.host_v[start:start + nb].view(torch.int16).numpy().copy()
        self.mirror[rid] = [k.transpose(1, 0, 2, 3).reshape(k.shape[1], nb * BS, -1)[:, :L].copy(),
                            v.transpose(1, 0, 2, 3).reshape(v.shape[1], nb * BS, -1)[:, :L].copy()]

    # ---- one decode iteration: append the new token's k, v, then attend over kv_len + 1 tokens
    def iterate(self, rows, lens, it):
        torch = self.torch
        sim = self.sim
        B = len(lens)
        self.bt_pin[:B].copy_(torch.from_numpy(sim.bt_all[rows]))
        self.dl_pin[:B].copy_(torch.from_numpy(lens))
        self.bt_dev[:B].copy_(self.bt_pin[:B], non_blocking=True)
        self.dl_dev[:B].copy_(self.dl_pin[:B], non_blocking=True)
        q, out = self.q_all[:B], self.out_all[:B]
        bt, dl = self.bt_dev[:B], self.dl_dev[:B]
        grown = lens + 1
        params = als.attn_params(q, self.dev_k, bt, out)
        need = als.decode_attention_workspace(params, int(grown.sum()))
        if self.ws is None or self.ws.numel() < need:
            self.ws = torch.empty(int(need * 1.5), dtype=torch.uint8, device="cuda")
        self.knew[:B].normal_(generator=self.gen)
        self.vnew[:B].normal_(generator=self.gen)
        e0, e1, e2 = self.ev[it % 2]
        e0.record()
        als.kv_append(self.knew[:B], self.vnew[:B], self.dev_k, self.dev_v, bt, dl)
        e1.record()
        als.decode_attention(q, self.dev_k, self.dev_v, bt, dl, out, kv_lens_host=grown, workspace=self.ws,
                             params=params)
        e2.record()
        # the scheduler runs on the iteration's result (sampled tokens): wait for THIS iteration only --
        # a device-wide synchronisation would also wait for the prefetch copies on the side stream
        e2.synchronize()
        # schedule gap: end of the previous iteration's attention -> start of this iteration's work
        # on the compute stream (host scheduling, plus any wait for copies that were not finished)
        prev = self.ev[(it + 1) % 2][2] if it > 0 else None
        timing = dict(attn_us=e1.elapsed_time(e2) * 1e3, fwd_us=e0.elapsed_time(e2) * 1e3,
                      gap_us=prev.elapsed_time(e0) * 1e3 if prev is not None else None)
        if sim.cfg.verify_every:
            kn = self.knew[:B].view(torch.int16).cpu().numpy()
            vn = self.vnew[:B].view(torch.int16).cpu().numpy()
            for i, r in enumerate(sim.run_ids):
                m = self.mirror[int(r)]
                m[0] = np.concatenate([m[0], kn[i][:, None, :]], axis=1)
                m[1] = np.concatenate([m[1], vn[i][:, None, :]], axis=1)
            if it % sim.cfg.verify_every == 0:
                self.verify(sim.run_ids, grown)
        return timing

    def verify(self, ids, lens):
        torch = self.torch
        for i, r in enumerate(ids):
            r = int(r)
            L = int(lens[i])
            blk = torch.tensor(self.sim.blocks_of[r], dtype=torch.int64, device="cuda")
            k = self.dev_k.index_select(0, blk).view(torch.int16).cpu().numpy()
            v = self.dev_v.index_select(0, blk).view(torch.int16).cpu().numpy()
            k = k.transpose(1, 0, 2, 3).reshape(k.shape[1], -1, k.shape[3])[:, :L]
            v = v.transpose(1, 0, 2, 3).reshape(v.shape[1], -1, v.shape[3])[:, :L]
            if not (np.array_equal(k, self.mirror[r][0]) and np.array_equal(v, self.mirror[r][1])):
                raise AssertionError(f"device KV of request {r} differs from the host mirror")

    def finish(self, stats):
        self.torch.cuda.synchronize()
        for kind in ("h2d_prefetch", "h2d_critical", "d2h"):
            ms = sum(a.elapsed_time(b) for a, b, _, k in self.copy_events if k == kind)
            by = sum(n for _, _, n, k in self.copy_events if k == kind)
            stats[kind + "_bytes"] = int(by)
            stats[kind + "_ms"] = float(ms)
        self.pipe.destroy()
        als.stage_set_policy(als.STAGE_AUTO)


class DecodeSim:
    def __init__(self, prefix_lens, output_lens, cfg: SimConfig):
        self.cfg = cfg
        self.n = len(prefix_lens)
        self.prefix = np.asarray(prefix_lens, dtype=np.int32)
        self.out_len = np.asarray(output_lens, dtype=np.int32)
        Hkv, D = cfg.num_kv_heads, cfg.head_dim
        self.block_bytes = Hkv * BS * D * 2
        self.max_len = int((self.prefix + self.out_len).max())
        self.MB = (self.max_len + BS - 1) // BS + 1
        self.b_max = max(int(cfg.b_max_frac * cfg.hbm_blocks), 1)
        self.cand_blocks = cfg.cand_blocks or self.b_max + 2 * self.MB
        # one physical pool: the scheduler's budget, the candidate budget, and room for blocks
        # whose eviction copy is still in flight
        self.pool_blocks = cfg.hbm_blocks + self.cand_blocks + 2 * self.MB
        self.free_blocks: List[int] = list(range(self.pool_blocks - 1, -1, -1))
        self.owner = np.full(self.pool_blocks, -1, dtype=np.int64)     # request that holds each block
        nblk = (self.prefix.astype(np.int64) + BS - 1) // BS
        self.host_start = np.concatenate([[0], np.cumsum(nblk)[:-1]])
        self.arena = cfg.host_arena_blocks or int(nblk.sum())
        self.evict_slots = cfg.evict_slots or cfg.max_batch * 2
        self.evict_free = list(range(self.evict_slots - 1, -1, -1))
        self.evicted: Dict[int, Tuple[int, int, int]] = {}        # rid -> (host slot, blocks, kv_len)
        self.blocks_of: Dict[int, List[int]] = {}                 # running requests
        self.prefetched: Dict[int, Tuple[int, List[int]]] = {}    # rid -> (copy group, blocks): staged, not admitted
        self.cand_used = 0
        self.cur_len: Dict[int, int] = {}                         # tokens in the device cache
        self.row_of: Dict[int, int] = {}
        self.rows_free = list(range(4 * cfg.max_batch + 64 - 1, -1, -1))
        self.bt_all = np.full((len(self.rows_free), self.MB), -1, dtype=np.int32)
        self.pending_free: List[Tuple[object, List[int]]] = []    # (eviction-copy event, blocks)
        self.b_cand: List[int] = []                               # mirrors of the scheduler's two buffers
        self.r_cand: List[int] = []
        self.sched = als.Scheduler(cfg.hbm_blocks, BS, cfg.max_batch)
        self.tree = None
        self.waiting = list(range(self.n))                        # arrival order
        if cfg.policy == "aligned":
            self.tree = als.QuadTree(65536, 16)
            for r in range(self.n):
                self.tree.insert(r, int(self.prefix[r]), int(nblk[r]))
        self.origin = 0
        self.iteration = 0                                        # decode iterations done: the loop's clock
        self.first_admitted: Dict[int, int] = {}                  # rid -> iteration of its first admission
        self.run_ids = np.zeros(0, dtype=np.int32)
        self.stats = dict(attn_us=[], fwd_us=[], gap_us=[], batch_size=[], tokens=[], sched_ms=[], switching=0,
                          evictions=0, admissions=0, admitted_prefetched=0, admitted_resident=0, completed=0, restored_blocks=0,
                          evicted_blocks=0, eviction_lens=[])
        self.be = _DryBackend(self) if cfg.dry else _GpuBackend(self)

    # ------------------------------------------------------------------ batches
    def _next_candidate_batch(self) -> bool:
        cfg = self.cfg
        if self.tree is not None:
            if len(self.tree) == 0:
                return False
            ids, _ = self.tree.next_batch(self.b_max, cfg.k_min, now=float(self.iteration),
                                          starve_after=None if cfg.starve_after < 0 else cfg.starve_after)
        else:
            if not self.waiting:
                return False
            ids, self.waiting = self.waiting[:cfg.max_batch], self.waiting[cfg.max_batch:]
        ids = np.asarray(ids, dtype=np.int32)
        self.sched.push_candidate_batch(self.origin, ids, self.prefix[ids], self.out_len[ids])
        self.b_cand.extend(int(i) for i in ids)
        self.origin += 1
        return True

    # ------------------------------------------------------------------ blocks
    def _reclaim(self, wait: bool):
        """Blocks of evicted requests come back when their copy to the host has finished."""
        while self.pending_free:
            ev, blocks = self.pending_free[0]
            if not ev.query():
                if not wait:
                    return
                ev.synchronize()
            self.pending_free.pop(0)
            self.free_blocks.extend(blocks)
            wait = False

    def _alloc(self, n: int, rid: int) -> List[int]:
        while len(self.free_blocks) < n:
            if not self.pending_free:
                raise RuntimeError("decode simulation: HBM block pool exhausted")
            self._reclaim(wait=True)
        got = [self.free_blocks.pop() for _ in range(n)]
        assert (self.owner[got] == -1).all(), "a block was handed out twice"
        self.owner[got] = rid
        return got

    def _release(self, blocks: List[int], deferred=None):
        self.owner[blocks] = -1
        if deferred is None:
            self.free_blocks.extend(blocks)
        else:
            self.pending_free.append((deferred, blocks))

    def _row(self, rid: int, blocks: List[int]):
        row = self.rows_free.pop()
        self.row_of[rid] = row
        self.bt_all[row] = -1                 # unused columns hold an invalid id
        self.bt_all[row, :len(blocks)] = blocks

    # ------------------------------------------------------------------ data movement
    def _source(self, rid: int):
        """(arena, first host block, blocks, kv_len) of a request that is not in HBM."""
        if rid in self.evicted:
            slot, nb, L = self.evicted[rid]
            return "evict", slot * self.MB, nb, L
        L = int(self.prefix[rid])
        nb = (L + BS - 1) // BS
        start = int(self.host_start[rid])
        if self.cfg.host_arena_blocks:
            start %= max(self.arena - nb, 1)
        return "host", start, nb, L

    def _stage_group(self, rids: List[int], critical: bool) -> int:
        """One copy group on the side stream: at most one as_stage_kv call per host arena."""
        tick = self.be.begin_group()
        per_arena: Dict[str, Tuple[list, list]] = {}
        total = 0
        placed = []
        for rid in rids:
            arena, start, nb, L = self._source(rid)
            dst = self._alloc(nb, rid)
            s, d = per_arena.setdefault(arena, ([], []))
            s.append(np.arange(nb, dtype=np.int64) + start)
            d.append(np.asarray(dst, dtype=np.int32))
            total += nb
            placed.append((rid, dst, arena, start, nb, L))
        for arena, (s, d) in per_arena.items():
            self.be.stage(arena, np.concatenate(s), np.concatenate(d))
        self.be.end_group(tick, 2 * total * self.block_bytes, critical)
        for rid, dst, arena, start, nb, L in placed:
            if arena == "evict":
                slot, nb_e, _ = self.evicted.pop(rid)
                assert nb_e == nb
                self.evict_free.append(slot)
                self.stats["restored_blocks"] += nb
            else:
                self.cur_len[rid] = L
                self.be.make_mirror(rid, start, nb, L)
            self.prefetched[rid] = (tick, dst)
            self.cand_used += nb
        return tick

    def _prefetch_tick(self):
        """Stage what Algorithm 2 will admit next, in its order (candidate requests first, then
        the candidate batch), as far as the candidate budget and the free blocks reach."""
        # Short groups, at most two in flight: the side stream is a FIFO, and an eviction or a copy
        # that an admission waits for must not queue behind tens of milliseconds of prefetch.
        if self.be.outstanding() >= self.cfg.prefetch_groups_in_flight:
            return
        picks, need = [], 0
        for rid in self.r_cand + self.b_cand:
            if rid in self.prefetched:
                continue
            nb = self._source(rid)[2]
            if self.cand_used + need + nb > self.cand_blocks or len(self.free_blocks) < need + nb:
                break
            if picks and need + nb > self.cfg.prefetch_group_blocks:
                break
            picks.append(rid)
            need += nb
        if picks:
            self._stage_group(picks, critical=False)

    def _admit(self, rids: List[int]):
        late = [r for r in rids if r not in self.prefetched]
        if late:                                   # not staged ahead: the copy is on the critical path
            self._stage_group(late, critical=True)
        ticks = {}
        for rid in rids:
            tick, blocks = self.prefetched.pop(rid)
            self.cand_used -= len(blocks)
            ticks[tick] = ticks.get(tick, 0) + (0 if rid in late else 1)
            self.blocks_of[rid] = blocks           # admission itself: the blocks change owner
            self.first_admitted.setdefault(rid, self.iteration)
            self._row(rid, blocks)
            (self.b_cand if rid in self.b_cand else self.r_cand).remove(rid)
            self.stats["admissions"] += 1
            self.stats["admitted_prefetched"] += 0 if rid in late else 1
        for tick, n_ahead in ticks.items():
            # the compute stream waits for those copies if they are still running
            if self.be.acquire(tick):
                self.stats["admitted_resident"] += n_ahead

    def _evict(self, rid: int):
        blocks = self.blocks_of.pop(rid)
        L = self.cur_len[rid]
        assert len(blocks) == (L + BS - 1) // BS, "evicted request's blocks do not match its length"
        if not self.evict_free:
            raise RuntimeError("decode simulation: no host slot left for an evicted request (raise evict_slots)")
        slot = self.evict_free.pop()
        self.evicted[rid] = (slot, len(blocks), L)
        dst = np.arange(len(blocks), dtype=np.int64) + slot * self.MB
        ev = self.be.unstage_behind_event(dst, np.asarray(blocks, dtype=np.int32),
                                          2 * len(blocks) * self.block_bytes)
        self._release(blocks, deferred=ev)         # reusable once the copy has finished
        self.rows_free.append(self.row_of.pop(rid))
        self.r_cand.append(rid)
        self.stats["evictions"] += 1
        self.stats["evicted_blocks"] += len(blocks)
        self.stats["eviction_lens"].append(L)

    # ------------------------------------------------------------------ main loop
    def run(self, max_iters: int = 100000):
        cfg = self.cfg
        first = True
        it = 0
        for _ in range(max_iters):
            t_s = time.perf_counter()
            if self.sched.state()["candidate_batch"] == 0:
                self._next_candidate_batch()
            done, evicted, admitted, case = self.sched.step(advance=not first)
            first = False
            for r in done:
                self._release(self.blocks_of.pop(r))
                self.rows_free.append(self.row_of.pop(r))
                self.cur_len.pop(r, None)
                if not cfg.dry:
                    self.be.mirror.pop(r, None)
                self.stats["completed"] += 1
            for r in evicted:
                self._evict(r)
            self._reclaim(wait=False)
            if admitted:
                self._admit(admitted)
            if cfg.prefetch:
                self._prefetch_tick()
            ids, lens, origins = self.sched.running()
            if len(ids) == 0:
                st = self.sched.state()
                if st["candidate_batch"] == 0 and st["candidate_requests"] == 0 and not self._next_candidate_batch():
                    break
                continue
            # the new token of every request goes to position kv_len: a fresh block where that starts one
            rows = np.empty(len(ids), dtype=np.int64)
            for i, r in enumerate(ids):
                r = int(r)
                assert self.cur_len[r] == int(lens[i]), "scheduler and device lengths differ"
                if lens[i] % BS == 0:
                    blk = self._alloc(1, r)[0]
                    self.blocks_of[r].append(blk)
                    self.bt_all[self.row_of[r], len(self.blocks_of[r]) - 1] = blk
                rows[i] = self.row_of[r]
            self.run_ids = ids
            self.stats["sched_ms"].append((time.perf_counter() - t_s) * 1e3)
            timing = self.be.iterate(rows, np.ascontiguousarray(lens), it)
            for r in ids:
                self.cur_len[int(r)] += 1
            if timing is not None:
                self.stats["attn_us"].append(timing["attn_us"])
                self.stats["fwd_us"].append(timing["fwd_us"])
                if timing["gap_us"] is not None:
                    self.stats["gap_us"].append(timing["gap_us"])
            self.stats["batch_size"].append(len(ids))
            self.stats["tokens"].append(int(lens.sum()) + len(ids))
            if len(set(origins.tolist())) > 1:
                self.stats["switching"] += 1
            it += 1
            self.iteration = it
        self._reclaim(wait=True)
        self.stats["wait_iterations"] = [self.first_admitted[r] for r in sorted(self.first_admitted)]
        self.be.finish(self.stats)
        return self.stats


def _pct(a, q):
    return round(float(np.percentile(a, q)), 1)


def summarize(stats) -> dict:
    n_it = len(stats["batch_size"])
    if n_it == 0:
        return {"iterations": 0}
    gen_tokens = int(np.sum(stats["batch_size"]))
    out = {
        "iterations": n_it, "generated_tokens": gen_tokens,
        "mean_batch": round(float(np.mean(stats["batch_size"])), 1),
        "switching_iterations_pct": round(100.0 * stats["switching"] / n_it, 2),
        "evictions": stats["evictions"], "admissions": stats["admissions"],
        "admitted_staged_ahead": stats["admitted_prefetched"], "admitted_already_in_hbm": stats["admitted_resident"],
        "completed": stats["completed"],
        "host_sched_ms_mean": round(float(np.mean(stats["sched_ms"])), 3),
    }
    if stats.get("wait_iterations"):
        w = np.asarray(stats["wait_iterations"])
        out.update({"wait_iterations_p50": _pct(w, 50), "wait_iterations_p99": _pct(w, 99),
                    "wait_iterations_max": int(w.max())})
    if stats["attn_us"]:
        us = np.asarray(stats["attn_us"])
        fwd = np.asarray(stats["fwd_us"])
        gap = np.asarray(stats["gap_us"]) if stats["gap_us"] else np.zeros(1)
        total_us = float(fwd.sum() + gap.sum())
        out.update({
            "attn_us_mean": round(float(us.mean()), 1), "attn_us_p50": _pct(us, 50), "attn_us_p90": _pct(us, 90),
            "attn_us_p99": _pct(us, 99),
            "schedule_gap_us_p50": _pct(gap, 50), "schedule_gap_us_p90": _pct(gap, 90),
            "schedule_gap_us_p99": _pct(gap, 99), "schedule_gap_us_max": _pct(gap, 100),
            "schedule_gap_us_mean": round(float(gap.mean()), 1),
            "gap_share_of_time_pct": round(100.0 * float(gap.sum()) / total_us, 1),
            "tokens_per_s": round(gen_tokens / (total_us * 1e-6), 0),
            "attn_tokens_per_s": round(gen_tokens / (us.sum() * 1e-6), 0),
        })
        for kind, label in (("h2d_prefetch", "staged_ahead"), ("h2d_critical", "staged_at_admission"),
                            ("d2h", "unstaged")):
            by, ms = stats.get(kind + "_bytes", 0), stats.get(kind + "_ms", 0.0)
            out[label + "_GB"] = round(by / 1e9, 3)
            out[label + "_GBs"] = round(by / ms / 1e6, 1) if ms > 0 else None
    return out
