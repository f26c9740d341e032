"""fp64 oracle for batched decode-iteration attention over a paged KV cache.

TEST INFRASTRUCTURE ONLY: slow, obviously-correct NumPy; shares no code with
the HIP library and is never used by the product path.

What it computes is the plain definition of the paper's Section 2.2, Eq. 2:
for the newest token's query q and the request's cached keys / values
K = {k_1..k_n}, V = {v_1..v_n},

    Attention(q, K, V) = softmax(q K^T / sqrt(d_k)) V .

Readings taken where the paper is silent (all listed in the design notes):
  * d_k is the per-head dimension D; scale = 1/sqrt(D) unless overridden.
  * kv_len counts every cached token including the newest one; one query
    sees all kv_len rows (no causal mask; only rows >= kv_len are excluded).
  * grouped-query attention: query head h reads KV head h // G with
    G = num_q_heads / num_kv_heads (contiguous groups).
  * paged storage [num_blocks][num_kv_heads][block_size][D]; logical token t
    of request b is row t % bs of physical block block_table[b, t // bs];
    storage rows past kv_len and unused table entries never matter.

Parity pins (tests/test_oracle_attention.py): single-token KV returns v_1;
identical keys give the mean of V; permutation of KV positions; key-shift
invariance incl. a 1e4 score offset; one-hot limit; convex-hull bound; a
closed-form case with rational softmax weights (tests/golden); agreement with
torch's scaled_dot_product_attention in float64; GQA == MHA on replicated KV
heads; physical-placement and poisoned-padding invariance; the split-KV merge
identity.
"""
from __future__ import annotations

import math

import numpy as np


def gather_kv(blocks: np.ndarray, block_table_row: np.ndarray, kv_len: int, kv_head: int) -> np.ndarray:
    """Logical [kv_len][D] fp64 matrix of one request / KV head, read through
    the block table (paged-storage reading above)."""
    bs = blocks.shape[2]
    nb = (int(kv_len) + bs - 1) // bs
    rows = [np.asarray(blocks[int(block_table_row[j]), kv_head], dtype=np.float64) for j in range(nb)]
    return np.concatenate(rows, axis=0)[: int(kv_len)]


def attention_single(q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float) -> np.ndarray:
    """Eq. 2 for one query vector: softmax(scale * K q) V, all in fp64."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    s = (K @ q) * scale
    p = np.exp(s - s.max())
    return (p @ V) / p.sum()


def decode_attention(q, k_blocks, v_blocks, block_table, kv_lens, scale=None) -> np.ndarray:
    """Eq. 2 for every (request, query head) of a batch; returns fp64 [B][H_q][D].

    q           : [B][H_q][D] float array (any float dtype; widened to fp64)
    k_blocks    : [NB][H_kv][bs][D]
    v_blocks    : [NB][H_kv][bs][D]
    block_table : int [B][MB]
    kv_lens     : int [B], every entry >= 1
    """
    q = np.asarray(q)
    B, Hq, D = q.shape
    Hkv = k_blocks.shape[1]
    if Hq % Hkv:
        raise ValueError("num_q_heads must be a multiple of num_kv_heads")
    G = Hq // Hkv
    sc = 1.0 / math.sqrt(D) if scale is None else float(scale)
    out = np.zeros((B, Hq, D), dtype=np.float64)
    for b in range(B):
        L = int(kv_lens[b])
        if L < 1:
            raise ValueError("softmax over an empty KV set is undefined")
        for g in range(Hkv):
            K = gather_kv(k_blocks, block_table[b], L, g)
            V = gather_kv(v_blocks, block_table[b], L, g)
            for h in range(g * G, (g + 1) * G):
                out[b, h] = attention_single(q[b, h], K, V, sc)
    return out


def merge_partials(ms, ls, accs) -> np.ndarray:
    """Exact merge of split-KV partial results (the re-association the
    split-KV kernel relies on).  Part i covers a disjoint subset S_i of the
    KV positions and carries m_i = max_{t in S_i} s_t,
    l_i = sum exp(s_t - m_i), acc_i = sum exp(s_t - m_i) v_t.  With
    M = max_i m_i the attention over the union is
        sum_i e^{m_i - M} acc_i / sum_i e^{m_i - M} l_i .
    """
    ms = np.asarray(ms, dtype=np.float64)
    ls = np.asarray(ls, dtype=np.float64)
    accs = np.asarray(accs, dtype=np.float64)
    w = np.exp(ms - ms.max())
    return (w[:, None] * accs).sum(axis=0) / (w * ls).sum()
