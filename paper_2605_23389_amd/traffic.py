"""Algorithmic byte / flop model of one decode-attention call.

From the paper's Table 1 (attention touches 2*s*h KV elements per generated
token and performs as many multiply-adds) and Section 3.2 (about 512 KB of KV
per token over all layers of Llama2-7B in 16-bit: 2 * 32 layers * 32 heads *
128 * 2 bytes).  Only real tokens count: no padded block rows, no
batch * longest-request padding.  With grouped-query attention a KV element
is counted once per KV head, not once per query head.
"""
from __future__ import annotations

import numpy as np


def kv_bytes_per_token(num_kv_heads: int, head_dim: int, elem_bytes: int, layers: int = 1) -> int:
    """K and V bytes of one cached token."""
    return 2 * layers * num_kv_heads * head_dim * elem_bytes


def attention_bytes(kv_lens, num_q_heads: int, num_kv_heads: int, head_dim: int,
                    elem_bytes: int = 2, out_bytes: int = 2, block_size: int = 16) -> int:
    """Bytes one decode_attention call must move for a batch (one layer):
    every K/V element of every real token once, q in, out out, the block-table
    entries and the lengths.  Split-KV partials are the kernel's own overhead
    and are not counted."""
    lens = np.asarray(kv_lens, dtype=np.int64)
    kv = int(lens.sum()) * kv_bytes_per_token(num_kv_heads, head_dim, elem_bytes)
    qo = int(lens.shape[0]) * num_q_heads * head_dim * (elem_bytes + out_bytes)
    meta = int(((lens + block_size - 1) // block_size).sum()) * 4 + int(lens.shape[0]) * 4
    return kv + qo + meta


def attention_flops(kv_lens, num_q_heads: int, head_dim: int) -> int:
    """2*D flops for q.k and 2*D for p.v per (token, query head)."""
    return int(np.asarray(kv_lens, dtype=np.int64).sum()) * num_q_heads * 4 * head_dim
