"""Device-resident synthetic workloads for benchmarks and full-size tests.

Only plumbing: allocates the paged K/V pools with PyTorch, fills them with
seeded N(0,1) values directly on the device (full-size pools are tens of GB,
too large to draw on the host), and assembles per-batch tensors.  No step of
the hot path is computed here.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

from . import workloads as wl


@dataclass
class DevicePool:
    k: "torch.Tensor"            # [NB][H_kv][16][D]
    v: "torch.Tensor"
    block_table: np.ndarray      # host int32 [n][MB], one row per request
    kv_lens: np.ndarray          # host int32 [n]
    num_q_heads: int
    num_kv_heads: int
    head_dim: int


def make_device_pool(kv_lens, num_q_heads, num_kv_heads, head_dim, dtype="bf16", seed=0,
                     device="cuda:0", table_seed=None) -> DevicePool:
    """One shared pool holding every request's KV; block ids are a seeded
    permutation (random physical placement).  table_seed fixes the placement
    independently of the data (the layers of one model share a block table)."""
    import torch
    kv_lens = np.asarray(kv_lens, dtype=np.int32)
    bt, used = wl.build_block_table(kv_lens, seed=seed if table_seed is None else table_seed)
    tdt = {"bf16": torch.bfloat16, "fp16": torch.float16, "fp32": torch.float32}[dtype]
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    shape = (used, num_kv_heads, wl.BLOCK_SIZE, head_dim)
    pools = []
    for _ in range(2):
        t = torch.empty(shape, dtype=tdt, device=device)
        flat = t.view(-1)
        step = 1 << 28
        for i in range(0, flat.numel(), step):
            flat[i:i + step].normal_(generator=gen)
        pools.append(t)
    return DevicePool(k=pools[0], v=pools[1], block_table=bt, kv_lens=kv_lens,
                      num_q_heads=num_q_heads, num_kv_heads=num_kv_heads, head_dim=head_dim)


@dataclass
class DeviceBatch:
    members: np.ndarray          # request indices
    kv_lens_host: np.ndarray     # int32 [B]
    kv_lens: "torch.Tensor"
    block_table: "torch.Tensor"  # int32 [B][MB_batch]
    q: "torch.Tensor"
    out: "torch.Tensor"
    tokens: int


def make_device_batches(pool: DevicePool, order, offsets, seed=0, out_dtype=None) -> List[DeviceBatch]:
    """Per-batch device tensors for the grouping (order, offsets)."""
    import torch
    dev = pool.k.device
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed + 1)
    batches = []
    for j in range(len(offsets) - 1):
        members = np.asarray(order[offsets[j]:offsets[j + 1]], dtype=np.int64)
        lens = pool.kv_lens[members]
        mb = int((int(lens.max()) + wl.BLOCK_SIZE - 1) // wl.BLOCK_SIZE)
        bt = np.ascontiguousarray(pool.block_table[members, :mb])
        q = torch.empty((len(members), pool.num_q_heads, pool.head_dim), dtype=pool.k.dtype, device=dev)
        q.normal_(generator=gen)
        out = torch.empty_like(q, dtype=out_dtype or pool.k.dtype)
        batches.append(DeviceBatch(members=members, kv_lens_host=np.ascontiguousarray(lens),
                                   kv_lens=torch.from_numpy(np.ascontiguousarray(lens)).to(dev),
                                   block_table=torch.from_numpy(bt).to(dev), q=q, out=out,
                                   tokens=int(lens.sum())))
    return batches


def fetch_request_kv(pool: DevicePool, request: int):
    """Copy one request's blocks to the host (for sampled oracle checks):
    returns (k_blocks, v_blocks, block_table_row) re-indexed 0..nb-1, as
    float32 arrays."""
    import torch
    L = int(pool.kv_lens[request])
    nb = (L + wl.BLOCK_SIZE - 1) // wl.BLOCK_SIZE
    ids = torch.from_numpy(pool.block_table[request, :nb].astype(np.int64)).to(pool.k.device)
    k = pool.k.index_select(0, ids).float().cpu().numpy()
    v = pool.v.index_select(0, ids).float().cpu().numpy()
    return k, v, np.arange(nb, dtype=np.int32)


def fetch_request_head(pool: DevicePool, request: int, kv_head: int):
    """One request's logical K and V for one KV head as float32 [L][D] host
    arrays (sampled oracle checks on full-size pools)."""
    import torch
    L = int(pool.kv_lens[request])
    nb = (L + wl.BLOCK_SIZE - 1) // wl.BLOCK_SIZE
    ids = torch.from_numpy(pool.block_table[request, :nb].astype(np.int64)).to(pool.k.device)
    k = pool.k.index_select(0, ids)[:, kv_head].reshape(nb * wl.BLOCK_SIZE, -1)[:L].float().cpu().numpy()
    v = pool.v.index_select(0, ids)[:, kv_head].reshape(nb * wl.BLOCK_SIZE, -1)[:L].float().cpu().numpy()
    return k, v
