"""Seeded synthetic inputs for the decode-attention hot path.

This module only *draws inputs* (KV lengths, paged K/V pools, block tables,
queries, random groupings).  It contains none of the method's arithmetic: no
softmax, no dot products, no batching policy.  Both the HIP path and the CPU
oracle are fed from here so that they see bit-identical inputs; neither of
them is imported here.

Shapes stand in for the length-skewed serving traces the paper evaluates on
(Section 2.3, Figure 2: long-tailed prefix-length CDFs; Section 4.1: short
requests under one thousand tokens mixed with long ones up to eight
thousand).  The traces themselves are not available; lognormal / uniform
draws of the same character replace them.

Layout of the paged pool (the library's contract):
    k_blocks, v_blocks : [num_blocks][num_kv_heads][block_size][head_dim]
    block_table        : int32 [batch][max_blocks_per_seq]
    kv_lens            : int32 [batch]
Logical token t of request b lives in physical block block_table[b, t // bs],
row t % bs.  bf16 and fp16 tensors are carried in NumPy as uint16 bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BLOCK_SIZE = 16


# ----------------------------------------------------------------------------
# bf16 <-> fp32 bit-pattern helpers (input representation only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even), returned as uint16 bits.

    NaN stays NaN (quiet bit forced); +-Inf stays +-Inf.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = np.isnan(x)
    out = rounded.astype(np.uint16)
    if nan.any():
        out = np.where(nan, ((u >> np.uint32(16)) | np.uint32(0x0040)).astype(np.uint16), out)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to fp32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to IEEE binary16 (round-to-nearest-even), as uint16 bits."""
    with np.errstate(over="ignore"):
        return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of binary16 bit patterns (uint16) to fp32."""
    return np.ascontiguousarray(b, dtype=np.uint16).view(np.float16).astype(np.float32)


_TO_BITS = {"bf16": f32_to_bf16_bits, "fp16": f32_to_f16_bits}
_FROM_BITS = {"bf16": bf16_bits_to_f32, "fp16": f16_bits_to_f32}


# ----------------------------------------------------------------------------
# KV length draws
# ----------------------------------------------------------------------------
def lognormal_lengths(rng: np.random.Generator, n: int, median: float, sigma: float,
                      lo: int, hi: int) -> np.ndarray:
    """clip(rint(exp(ln(median) + sigma * N(0,1))), lo, hi) as int32."""
    z = rng.standard_normal(n)
    x = np.rint(np.exp(np.log(median) + sigma * z))
    return np.clip(x, lo, hi).astype(np.int32)


def uniform_lengths(rng: np.random.Generator, n: int, lo: int, hi: int) -> np.ndarray:
    """Uniform integers in [lo, hi] as int32."""
    return rng.integers(lo, hi + 1, n).astype(np.int32)


def random_grouping(n: int, batch_size: int, seed: int):
    """Length-oblivious comparison grouping: a seeded permutation cut into
    consecutive chunks of batch_size (the FCFS-like policy the paper compares
    prefix-aware batching against, Section 3.3 / Figure 12).  Returns
    (order int32[n], batch_offsets int32[nb+1])."""
    rng = np.random.default_rng(seed)
    order = rng.permutation(n).astype(np.int32)
    nb = (n + batch_size - 1) // batch_size
    offs = np.minimum(np.arange(nb + 1, dtype=np.int64) * batch_size, n).astype(np.int32)
    return order, offs


# ----------------------------------------------------------------------------
# Paged KV problem instances
# ----------------------------------------------------------------------------
@dataclass
class PagedBatch:
    """One decode-iteration attention problem over a paged KV pool.

    q, k_blocks, v_blocks are float32 arrays when dtype == "fp32" and uint16
    bit patterns when dtype is "bf16" or "fp16".
    """
    dtype: str
    q: np.ndarray            # [B][H_q][D]
    k_blocks: np.ndarray     # [NB][H_kv][bs][D]
    v_blocks: np.ndarray     # [NB][H_kv][bs][D]
    block_table: np.ndarray  # int32 [B][MB]
    kv_lens: np.ndarray      # int32 [B]
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_size: int = BLOCK_SIZE
    meta: dict = field(default_factory=dict)

    @property
    def batch(self) -> int:
        return int(self.kv_lens.shape[0])

    @property
    def num_blocks(self) -> int:
        return int(self.k_blocks.shape[0])

    def as_float(self, name: str) -> np.ndarray:
        """q / k_blocks / v_blocks widened to a float array (exact)."""
        a = getattr(self, name)
        return _FROM_BITS[self.dtype](a) if self.dtype in _FROM_BITS else a


def _draw_tensor(rng, shape, dtype):
    x = rng.standard_normal(shape, dtype=np.float32)
    return _TO_BITS[dtype](x) if dtype in _TO_BITS else x


def poison_value(dtype: str, kind: str):
    """Bit pattern / value used to fill storage no result may depend on."""
    table = {"nan": np.float32(np.nan), "inf": np.float32(np.inf),
             "ninf": np.float32(-np.inf), "big": np.float32(1e30), "zero": np.float32(0)}
    v = np.asarray([table[kind]], dtype=np.float32)
    return _TO_BITS[dtype](v)[0] if dtype in _TO_BITS else v[0]


def make_paged_batch(kv_lens, num_q_heads: int, num_kv_heads: int, head_dim: int,
                     dtype: str = "bf16", seed: int = 0, block_size: int = BLOCK_SIZE,
                     spare_blocks: int = 0, poison: Optional[str] = None,
                     extra_table_cols: int = 0) -> PagedBatch:
    """Draw q, K, V ~ N(0,1) for the given KV lengths and scatter K/V into a
    paged pool through a random permutation of physical block ids.

    spare_blocks : additional pool blocks owned by nobody.
    poison       : None -> padding rows, spare blocks and unused table entries
                   are zero / block 0; otherwise one of "nan", "inf", "ninf",
                   "big": every storage row past a request's kv_len and every
                   spare block is filled with it, and unused block_table
                   entries point at a spare (poisoned) block when one exists.
    """
    rng = np.random.default_rng(seed)
    kv_lens = np.asarray(kv_lens, dtype=np.int32)
    B = int(kv_lens.shape[0])
    nblk = (kv_lens.astype(np.int64) + block_size - 1) // block_size
    used = int(nblk.sum())
    NB = used + int(spare_blocks)
    MB = int(nblk.max()) + int(extra_table_cols) if B else 1
    perm = rng.permutation(NB).astype(np.int32)

    shape = (NB, num_kv_heads, block_size, head_dim)
    k_blocks = _draw_tensor(rng, shape, dtype)
    v_blocks = _draw_tensor(rng, shape, dtype)
    q = _draw_tensor(rng, (B, num_q_heads, head_dim), dtype)

    fill_id = int(perm[used]) if NB > used else 0
    block_table = np.full((B, MB), fill_id if poison else 0, dtype=np.int32)
    cur = 0
    for b in range(B):
        n = int(nblk[b])
        block_table[b, :n] = perm[cur:cur + n]
        cur += n

    if poison:
        pv = poison_value(dtype, poison)
        for b in range(B):
            tail = int(kv_lens[b]) % block_size
            if tail:
                last = int(block_table[b, int(nblk[b]) - 1])
                k_blocks[last, :, tail:, :] = pv
                v_blocks[last, :, tail:, :] = pv
        for pid in perm[used:]:
            k_blocks[int(pid)] = pv
            v_blocks[int(pid)] = pv

    return PagedBatch(dtype=dtype, q=q, k_blocks=k_blocks, v_blocks=v_blocks,
                      block_table=block_table, kv_lens=kv_lens,
                      num_q_heads=num_q_heads, num_kv_heads=num_kv_heads,
                      head_dim=head_dim, block_size=block_size,
                      meta={"seed": seed, "poison": poison, "used_blocks": used})


def repage(pb: PagedBatch, seed: int) -> PagedBatch:
    """Same logical K/V, different physical placement: re-draw the block
    permutation and move the data accordingly."""
    rng = np.random.default_rng(seed)
    NB = pb.num_blocks
    perm = rng.permutation(NB).astype(np.int32)   # old id -> new id
    k2 = np.empty_like(pb.k_blocks)
    v2 = np.empty_like(pb.v_blocks)
    k2[perm] = pb.k_blocks
    v2[perm] = pb.v_blocks
    bt2 = perm[pb.block_table]
    return PagedBatch(dtype=pb.dtype, q=pb.q, k_blocks=k2, v_blocks=v2, block_table=bt2,
                      kv_lens=pb.kv_lens, num_q_heads=pb.num_q_heads,
                      num_kv_heads=pb.num_kv_heads, head_dim=pb.head_dim,
                      block_size=pb.block_size, meta=dict(pb.meta, repaged=seed))


# ----------------------------------------------------------------------------
# The benchmark configurations (lengths only; tensors are drawn separately so
# that full-size pools can be generated directly on the device)
# ----------------------------------------------------------------------------
def config_lengths(cfg: int, seed: int = 0) -> np.ndarray:
    """KV lengths of the numbered workload.

    0: 8 requests, U{16..256}                       (tiny parity case)
    1: 64 requests, lognormal(median 1024, s 0.8) clipped [128, 8192]
    2: 1024 requests, lognormal(median 1024, s 1.2) clipped [64, 32768]
    3: 128 requests, U{4096..32768}
    4: 4096 requests, lognormal(median 2048, s 0.8) clipped [128, 16384]
    """
    rng = np.random.default_rng(seed)
    if cfg == 0:
        return uniform_lengths(rng, 8, 16, 256)
    if cfg == 1:
        return lognormal_lengths(rng, 64, 1024.0, 0.8, 128, 8192)
    if cfg == 2:
        return lognormal_lengths(rng, 1024, 1024.0, 1.2, 64, 32768)
    if cfg == 3:
        return uniform_lengths(rng, 128, 4096, 32768)
    if cfg == 4:
        return lognormal_lengths(rng, 4096, 2048.0, 0.8, 128, 16384)
    raise ValueError(f"unknown config {cfg}")


CONFIG_SHAPES = {
    0: dict(num_q_heads=4, num_kv_heads=4, head_dim=64, dtype="fp32"),
    1: dict(num_q_heads=32, num_kv_heads=32, head_dim=128, dtype="bf16"),
    2: dict(num_q_heads=32, num_kv_heads=32, head_dim=128, dtype="bf16"),
    3: dict(num_q_heads=64, num_kv_heads=8, head_dim=128, dtype="bf16"),
    4: dict(num_q_heads=64, num_kv_heads=8, head_dim=128, dtype="bf16"),
}


def batcher_lengths_tiny(seed: int = 0) -> np.ndarray:
    """32 requests with lengths U{16..256} (batcher half of the tiny case)."""
    return uniform_lengths(np.random.default_rng(seed + 1000), 32, 16, 256)


def build_block_table(kv_lens, block_size: int = BLOCK_SIZE, seed: int = 0,
                      num_blocks: Optional[int] = None, max_blocks: Optional[int] = None):
    """Block table for many requests over one shared pool: request r owns
    ceil(L_r / bs) physical blocks taken consecutively from a seeded
    permutation of range(num_blocks).  Returns (block_table int32 [n][MB],
    used_blocks)."""
    kv_lens = np.asarray(kv_lens, dtype=np.int64)
    nblk = (kv_lens + block_size - 1) // block_size
    used = int(nblk.sum())
    NB = used if num_blocks is None else int(num_blocks)
    if NB < used:
        raise ValueError("pool smaller than the blocks requested")
    MB = int(nblk.max()) if max_blocks is None else int(max_blocks)
    perm = np.random.default_rng(seed).permutation(NB).astype(np.int32)
    bt = np.zeros((len(kv_lens), MB), dtype=np.int32)
    starts = np.concatenate([[0], np.cumsum(nblk)[:-1]])
    for r in range(len(kv_lens)):
        n = int(nblk[r])
        bt[r, :n] = perm[int(starts[r]):int(starts[r]) + n]
    return bt, used
