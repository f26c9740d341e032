"""Multi-iteration decode simulation that drives the real library calls.

Plumbing only: it owns the HBM block free-list, the pinned host KV pool and
the per-iteration batch tensors, and calls the library for every step of the
path -- batch generation (as_qtree_* / arrival order), scheduling
(as_sched_step, paper Algorithm 2), KV migration (as_stage_kv /
as_unstage_kv), attention (as_decode_attention) and KV append (as_kv_append).
Prompts, model weights and sampled tokens do not exist here: prefix lengths
and output lengths are synthetic, queries and new K/V rows are random.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional

import numpy as np

from . import binding as als
from . import workloads as wl


@dataclass
class SimConfig:
    num_q_heads: int = 32
    num_kv_heads: int = 32
    head_dim: int = 128
    max_batch: int = 64
    hbm_blocks: int = 16384          # decode instance's block pool
    policy: str = "aligned"          # "aligned" (quad-tree DFS) or "fcfs" (arrival order)
    k_min: int = 36                  # paper Section 4.1
    b_max_frac: float = 0.4          # paper Section 4.1: 40 % of the GPU blocks
    host_arena_blocks: int = 0       # 0 => one unique host block per logical block (verification runs)
    seed: int = 0
    verify_every: int = 0            # >0: compare device KV with a host mirror every n-th iteration
    evict_slots: int = 0             # host slots for evicted requests (0 => 2 * max_batch)


class DecodeSim:
    def __init__(self, prefix_lens, output_lens, cfg: SimConfig):
        import torch
        self.torch = torch
        self.cfg = cfg
        self.n = len(prefix_lens)
        self.prefix = np.asarray(prefix_lens, dtype=np.int32)
        self.out_len = np.asarray(output_lens, dtype=np.int32)
        Hkv, D = cfg.num_kv_heads, cfg.head_dim
        self.block_bytes = Hkv * 16 * D * 2
        self.max_len = int((self.prefix + self.out_len).max())
        self.MB = (self.max_len + 15) // 16 + 1
        dev = "cuda"
        self.dev_k = torch.zeros((cfg.hbm_blocks, Hkv, 16, D), dtype=torch.bfloat16, device=dev)
        self.dev_v = torch.zeros_like(self.dev_k)
        self.free_blocks: List[int] = list(range(cfg.hbm_blocks - 1, -1, -1))
        # host pool: request r owns logical blocks [start_r, start_r + nblk_r)
        nblk = (self.prefix.astype(np.int64) + 15) // 16
        self.host_start = np.concatenate([[0], np.cumsum(nblk)[:-1]])
        total = int(nblk.sum())
        self.arena = cfg.host_arena_blocks or total
        g = torch.Generator().manual_seed(cfg.seed)
        self.host_k = torch.empty((self.arena, Hkv, 16, D), dtype=torch.bfloat16, pin_memory=True)
        self.host_v = torch.empty_like(self.host_k, pin_memory=True)
        chunk = torch.randn((min(self.arena, 256), Hkv, 16, D), generator=g).to(torch.bfloat16)
        for t in (self.host_k, self.host_v):
            for i in range(0, self.arena, chunk.shape[0]):
                m = min(chunk.shape[0], self.arena - i)
                t[i:i + m].copy_(chunk[:m] if not cfg.verify_every else
                                 torch.randn((m, Hkv, 16, D), generator=g).to(torch.bfloat16))
        # eviction arena: one slot of MB blocks per running slot
        slots = cfg.evict_slots or cfg.max_batch * 2
        self.evict_k = torch.empty((slots * self.MB, Hkv, 16, D), dtype=torch.bfloat16, pin_memory=True)
        self.evict_v = torch.empty_like(self.evict_k, pin_memory=True)
        self.evict_free = list(range(slots - 1, -1, -1))
        self.evict_slot: Dict[int, int] = {}
        self.blocks_of: Dict[int, List[int]] = {}      # device block ids of resident requests
        self.cur_len: Dict[int, int] = {}
        self.sched = als.Scheduler(cfg.hbm_blocks, 16, cfg.max_batch)
        self.side = torch.cuda.Stream()
        self.tree = None
        self.waiting = list(range(self.n))             # arrival order
        if cfg.policy == "aligned":
            self.tree = als.QuadTree(65536, 16)
            for r in range(self.n):
                self.tree.insert(r, int(self.prefix[r]), int(nblk[r]))
        self.origin = 0
        self.gen = torch.Generator(device=dev).manual_seed(cfg.seed + 1)
        self.mirror: Dict[int, tuple] = {}
        self.stats = dict(iter_us=[], batch_size=[], tokens=[], switching=0, evictions=0, admissions=0,
                          completed=0, stage_bytes=0, unstage_bytes=0, sched_ms=[])

    # ------------------------------------------------------------------ batches
    def _next_candidate_batch(self) -> bool:
        cfg = self.cfg
        if self.tree is not None:
            if len(self.tree) == 0:
                return False
            ids, _ = self.tree.next_batch(int(cfg.b_max_frac * cfg.hbm_blocks), cfg.k_min)
        else:
            if not self.waiting:
                return False
            ids, self.waiting = self.waiting[:cfg.max_batch], self.waiting[cfg.max_batch:]
        ids = np.asarray(ids, dtype=np.int32)
        self.sched.push_candidate_batch(self.origin, ids, self.prefix[ids], self.out_len[ids])
        self.origin += 1
        return True

    # ------------------------------------------------------------------ data movement
    def _admit(self, rid: int):
        torch = self.torch
        L = self.cur_len.get(rid, int(self.prefix[rid]))
        nb = (L + 15) // 16
        dst = [self.free_blocks.pop() for _ in range(nb)]
        self.blocks_of[rid] = dst
        if rid in self.evict_slot:                      # comes back from the candidate-requests buffer
            slot = self.evict_slot.pop(rid)
            src = np.arange(nb, dtype=np.int64) + slot * self.MB
            als.stage_kv(self.evict_k, self.evict_v, src, self.dev_k, self.dev_v, np.asarray(dst, dtype=np.int32),
                         self.block_bytes, stream=self.side)
            self.evict_free.append(slot)
        else:
            self.cur_len[rid] = L
            start = int(self.host_start[rid])
            if self.cfg.host_arena_blocks:
                start %= max(self.arena - nb, 1)
            src = np.arange(nb, dtype=np.int64) + start
            als.stage_kv(self.host_k, self.host_v, src, self.dev_k, self.dev_v, np.asarray(dst, dtype=np.int32),
                         self.block_bytes, stream=self.side)
            if self.cfg.verify_every:
                k = self.host_k[start:start + nb].view(torch.int16).numpy().copy()
                v = self.host_v[start:start + nb].view(torch.int16).numpy().copy()
                self.mirror[rid] = [k.transpose(1, 0, 2, 3).reshape(k.shape[1], nb * 16, -1)[:, :L].copy(),
                                    v.transpose(1, 0, 2, 3).reshape(v.shape[1], nb * 16, -1)[:, :L].copy()]
        self.stats["stage_bytes"] += 2 * nb * self.block_bytes
        self.stats["admissions"] += 1

    def _evict(self, rid: int):
        blocks = self.blocks_of.pop(rid)
        if not self.evict_free:
            raise RuntimeError("decode simulation: no host slot left for an evicted request (raise evict_slots)")
        slot = self.evict_free.pop()
        self.evict_slot[rid] = slot
        dst = np.arange(len(blocks), dtype=np.int64) + slot * self.MB
        # the compute stream has finished with these blocks before the copy starts
        self.side.wait_stream(self.torch.cuda.current_stream())
        als.unstage_kv(self.evict_k, self.evict_v, dst, self.dev_k, self.dev_v,
                       np.asarray(blocks, dtype=np.int32), self.block_bytes, stream=self.side)
        self.side.synchronize()                        # blocks may be reused right away
        self.free_blocks.extend(blocks)
        self.stats["unstage_bytes"] += 2 * len(blocks) * self.block_bytes
        self.stats["evictions"] += 1

    # ------------------------------------------------------------------ main loop
    def run(self, max_iters: int = 100000):
        import time
        torch = self.torch
        cfg = self.cfg
        Hq, Hkv, D = cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim
        compute = torch.cuda.current_stream()
        q_all = torch.empty((cfg.max_batch, Hq, D), dtype=torch.bfloat16, device="cuda").normal_(generator=self.gen)
        out_all = torch.empty_like(q_all)
        knew = torch.empty((cfg.max_batch, Hkv, D), dtype=torch.bfloat16, device="cuda")
        vnew = torch.empty_like(knew)
        bt_host = np.zeros((cfg.max_batch, self.MB), dtype=np.int32)
        ws = None
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        first = True
        for it in range(max_iters):
            t_s = time.perf_counter()
            if self.sched.state()["candidate_batch"] == 0:
                self._next_candidate_batch()
            done, evicted, admitted, case = self.sched.step(advance=not first)
            first = False
            for r in done:
                self.free_blocks.extend(self.blocks_of.pop(r))
                self.cur_len.pop(r, None)
                self.mirror.pop(r, None)
                self.stats["completed"] += 1
            for r in evicted:
                self._evict(r)
            for r in admitted:
                self._admit(r)
            ids, lens, origins = self.sched.running()
            if len(ids) == 0:
                st = self.sched.state()
                if st["candidate_batch"] == 0 and st["candidate_requests"] == 0 and not self._next_candidate_batch():
                    break
                continue
            B = len(ids)
            # a fresh block for every request whose next token starts one
            for i, r in enumerate(ids):
                r = int(r)
                self.cur_len[r] = int(lens[i])
                if lens[i] % 16 == 0:
                    self.blocks_of[r].append(self.free_blocks.pop())
                blk = self.blocks_of[r]
                bt_host[i, :len(blk)] = blk
            bt = torch.from_numpy(bt_host[:B]).cuda()
            dl = torch.from_numpy(np.ascontiguousarray(lens)).cuda()
            compute.wait_stream(self.side)               # admissions' copies are complete
            self.stats["sched_ms"].append((time.perf_counter() - t_s) * 1e3)
            q, out = q_all[:B], out_all[:B]
            params = als.attn_params(q, self.dev_k, bt, out)
            need = als.decode_attention_workspace(params, int(lens.sum()))
            if ws is None or ws.numel() < need:
                ws = torch.empty(int(need * 1.5), dtype=torch.uint8, device="cuda")
            ev0.record()
            als.decode_attention(q, self.dev_k, self.dev_v, bt, dl, out, kv_lens_host=lens, workspace=ws,
                                 params=params)
            ev1.record()
            knew[:B].normal_(generator=self.gen)
            vnew[:B].normal_(generator=self.gen)
            als.kv_append(knew[:B], vnew[:B], self.dev_k, self.dev_v, bt, dl)
            torch.cuda.synchronize()
            self.stats["iter_us"].append(ev0.elapsed_time(ev1) * 1e3)
            self.stats["batch_size"].append(B)
            self.stats["tokens"].append(int(lens.sum()))
            if len(set(origins.tolist())) > 1:
                self.stats["switching"] += 1
            if cfg.verify_every:
                kn = knew[:B].view(torch.int16).cpu().numpy()
                vn = vnew[:B].view(torch.int16).cpu().numpy()
                for i, r in enumerate(ids):
                    m = self.mirror[int(r)]
                    m[0] = np.concatenate([m[0], kn[i][:, None, :]], axis=1)
                    m[1] = np.concatenate([m[1], vn[i][:, None, :]], axis=1)
                if it % cfg.verify_every == 0:
                    self._verify(ids, lens + 1)
        return self.stats

    def _verify(self, ids, lens):
        torch = self.torch
        for i, r in enumerate(ids):
            r = int(r)
            L = int(lens[i])
            blk = torch.tensor(self.blocks_of[r], dtype=torch.int64, device="cuda")
            k = self.dev_k.index_select(0, blk).view(torch.int16).cpu().numpy()
            v = self.dev_v.index_select(0, blk).view(torch.int16).cpu().numpy()
            k = k.transpose(1, 0, 2, 3).reshape(k.shape[1], -1, k.shape[3])[:, :L]
            v = v.transpose(1, 0, 2, 3).reshape(v.shape[1], -1, v.shape[3])[:, :L]
            if not (np.array_equal(k, self.mirror[r][0]) and np.array_equal(v, self.mirror[r][1])):
                raise AssertionError(f"device KV of request {r} differs from the host mirror")


def summarize(stats) -> dict:
    us = np.asarray(stats["iter_us"])
    if len(us) == 0:
        return {"iterations": 0}
    gen_tokens = int(np.sum(stats["batch_size"]))
    return {
        "iterations": int(len(us)), "generated_tokens": gen_tokens,
        "attn_us_mean": round(float(us.mean()), 1), "attn_us_p50": round(float(np.percentile(us, 50)), 1),
        "attn_us_p90": round(float(np.percentile(us, 90)), 1), "attn_us_p99": round(float(np.percentile(us, 99)), 1),
        "attn_tokens_per_s": round(gen_tokens / (us.sum() * 1e-6), 0),
        "mean_batch": round(float(np.mean(stats["batch_size"])), 1),
        "switching_iterations_pct": round(100.0 * stats["switching"] / len(us), 2),
        "evictions": stats["evictions"], "admissions": stats["admissions"], "completed": stats["completed"],
        "staged_GB": round(stats["stage_bytes"] / 1e9, 2), "unstaged_GB": round(stats["unstage_bytes"] / 1e9, 2),
        "host_sched_ms_mean": round(float(np.mean(stats["sched_ms"])), 3),
    }
