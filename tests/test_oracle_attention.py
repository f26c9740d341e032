"""Pins for the attention oracle: facts the mathematics (and the one closed
form we can write by hand) fix, chosen so that a plausible slip in the oracle
-- dropped scale, wrong sign in the exponent, missing max-subtraction,
transposed operand, wrong GQA mapping, off-by-one in the tail mask or in the
paging arithmetic -- fails at least one of them."""
import json
import math
import os

import numpy as np
import pytest

from oracle import attention as oa
from paper_2605_23389_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _contig_to_paged(K, V, bs=16, seed=0, poison=None):
    """Scatter one request's [L][H][D] K/V into a paged pool."""
    L, H, D = K.shape
    nb = (L + bs - 1) // bs
    rng = np.random.default_rng(seed)
    NB = nb + 3
    perm = rng.permutation(NB)
    fill = 0.0 if poison is None else poison
    kb = np.full((NB, H, bs, D), fill, dtype=np.float64)
    vb = np.full((NB, H, bs, D), fill, dtype=np.float64)
    for t in range(L):
        kb[perm[t // bs], :, t % bs, :] = K[t]
        vb[perm[t // bs], :, t % bs, :] = V[t]
    bt = np.full((1, nb + 2), perm[-1], dtype=np.int32)
    bt[0, :nb] = perm[:nb]
    return kb, vb, bt


def test_closed_form_rational_weights():
    g = json.load(open(os.path.join(GOLD, "attention_rational.json")))
    D = g["head_dim"]
    q = np.array(g["q"])
    K = np.array([[math.log(w)] + rest for w, rest in zip(g["w"], g["k_rest"])])
    V = np.array(g["v"])
    out = oa.attention_single(q, K, V, 1.0 / math.sqrt(D))
    np.testing.assert_allclose(out, g["expected"], rtol=0, atol=1e-14)
    # and through the paged / batched entry point (H=1)
    kb, vb, bt = _contig_to_paged(K[:, None, :], V[:, None, :])
    out2 = oa.decode_attention(q[None, None, :], kb, vb, bt, np.array([3]))
    np.testing.assert_allclose(out2[0, 0], g["expected"], rtol=0, atol=1e-14)
    # a wrong scale (1/d_k, or none) must not reproduce it
    assert np.abs(oa.attention_single(q, K, V, 1.0) - g["expected"]).max() > 1e-2
    assert np.abs(oa.attention_single(q, K, V, 1.0 / D) - g["expected"]).max() > 1e-2


def test_single_token_returns_v_exactly():
    rng = np.random.default_rng(1)
    K = rng.standard_normal((1, 2, 8))
    V = rng.standard_normal((1, 2, 8))
    q = rng.standard_normal((1, 2, 8))
    kb, vb, bt = _contig_to_paged(K, V, poison=np.nan)
    out = oa.decode_attention(q, kb, vb, bt, np.array([1]))
    assert np.array_equal(out[0], V[0])


def test_identical_keys_or_zero_query_give_mean_of_v():
    rng = np.random.default_rng(2)
    L, D = 37, 16
    V = rng.standard_normal((L, D))
    k = rng.standard_normal(D)
    q = rng.standard_normal(D)
    out = oa.attention_single(q, np.tile(k, (L, 1)), V, 0.25)
    np.testing.assert_allclose(out, V.mean(axis=0), atol=1e-13)
    out0 = oa.attention_single(np.zeros(D), rng.standard_normal((L, D)), V, 0.25)
    np.testing.assert_allclose(out0, V.mean(axis=0), atol=1e-13)


def test_permuting_kv_positions_changes_nothing():
    rng = np.random.default_rng(3)
    L, D = 50, 32
    K, V, q = rng.standard_normal((L, D)), rng.standard_normal((L, D)), rng.standard_normal(D)
    p = rng.permutation(L)
    a = oa.attention_single(q, K, V, 1 / math.sqrt(D))
    b = oa.attention_single(q, K[p], V[p], 1 / math.sqrt(D))
    np.testing.assert_allclose(a, b, atol=1e-13)
    # permuting keys WITHOUT values must change it (catches K/V mix-ups)
    c = oa.attention_single(q, K[p], V, 1 / math.sqrt(D))
    assert np.abs(a - c).max() > 1e-3


def test_key_shift_invariance_and_large_offset():
    rng = np.random.default_rng(4)
    L, D = 40, 16
    K, V, q = rng.standard_normal((L, D)), rng.standard_normal((L, D)), rng.standard_normal(D)
    sc = 1 / math.sqrt(D)
    a = oa.attention_single(q, K, V, sc)
    c = rng.standard_normal(D)
    np.testing.assert_allclose(oa.attention_single(q, K + c, V, sc), a, atol=1e-12)
    # shift every score by +1e4: without max-subtraction exp overflows
    big = q * (1e4 / sc / (q @ q))
    assert abs((big @ q) * sc - 1e4) < 1e-6
    out = oa.attention_single(q, K + big, V, sc)
    assert np.isfinite(out).all()
    np.testing.assert_allclose(out, a, atol=1e-8)


def test_one_hot_limit_and_convex_hull():
    rng = np.random.default_rng(5)
    L, D = 33, 8
    K, V, q = rng.standard_normal((L, D)), rng.standard_normal((L, D)), rng.standard_normal(D)
    sc = 1 / math.sqrt(D)
    out = oa.attention_single(q, K, V, sc)
    assert (out <= V.max(axis=0) + 1e-15).all() and (out >= V.min(axis=0) - 1e-15).all()
    K2 = K.copy()
    K2[17] = q * (200.0 / sc / (q @ q)) + K[17]
    np.testing.assert_allclose(oa.attention_single(q, K2, V, sc), V[17], atol=1e-12)


def test_hand_softmax_two_keys():
    # scores 0 and ln 3 (scale 1) -> weights 1/4, 3/4
    q = np.array([1.0, 0.0])
    K = np.array([[0.0, 5.0], [math.log(3.0), -2.0]])
    V = np.array([[4.0, 0.0], [0.0, 4.0]])
    np.testing.assert_allclose(oa.attention_single(q, K, V, 1.0), [1.0, 3.0], atol=1e-14)


def test_matches_torch_sdpa_float64():
    torch = pytest.importorskip("torch")
    pb = wl.make_paged_batch(wl.uniform_lengths(np.random.default_rng(7), 5, 1, 90),
                             num_q_heads=4, num_kv_heads=4, head_dim=32, dtype="fp32", seed=7,
                             spare_blocks=2, poison="nan")
    out = oa.decode_attention(pb.q, pb.k_blocks, pb.v_blocks, pb.block_table, pb.kv_lens)
    for b in range(pb.batch):
        L = int(pb.kv_lens[b])
        for h in range(4):
            K = oa.gather_kv(pb.k_blocks, pb.block_table[b], L, h)
            V = oa.gather_kv(pb.v_blocks, pb.block_table[b], L, h)
            ref = torch.nn.functional.scaled_dot_product_attention(
                torch.tensor(pb.q[b, h], dtype=torch.float64)[None, None, None, :],
                torch.tensor(K)[None, None], torch.tensor(V)[None, None])
            np.testing.assert_allclose(out[b, h], ref[0, 0, 0].numpy(), atol=1e-12)


def test_gather_follows_block_table():
    # token t must come from block_table[t // bs], row t % bs -- brute force
    bs, D, H = 16, 4, 2
    L = 45
    K = np.arange(L * H * D, dtype=np.float64).reshape(L, H, D)
    kb, _, bt = _contig_to_paged(K, K, bs=bs, seed=11, poison=-1.0)
    for h in range(H):
        got = oa.gather_kv(kb, bt[0], L, h)
        assert np.array_equal(got, K[:, h, :])
    assert oa.gather_kv(kb, bt[0], 16, 0).shape == (16, D)
    assert oa.gather_kv(kb, bt[0], 17, 0).shape == (17, D)


def test_gqa_equals_mha_on_replicated_kv_heads():
    lens = np.array([19, 64, 5], dtype=np.int32)
    pb = wl.make_paged_batch(lens, num_q_heads=8, num_kv_heads=2, head_dim=16, dtype="fp32", seed=9)
    out = oa.decode_attention(pb.q, pb.k_blocks, pb.v_blocks, pb.block_table, pb.kv_lens)
    k_rep = np.repeat(pb.k_blocks, 4, axis=1)
    v_rep = np.repeat(pb.v_blocks, 4, axis=1)
    out_mha = oa.decode_attention(pb.q, k_rep, v_rep, pb.block_table, pb.kv_lens)
    np.testing.assert_array_equal(out, out_mha)
    # interleaved (h % H_kv) mapping would differ
    k_bad = np.tile(pb.k_blocks, (1, 4, 1, 1))
    v_bad = np.tile(pb.v_blocks, (1, 4, 1, 1))
    assert np.abs(oa.decode_attention(pb.q, k_bad, v_bad, pb.block_table, pb.kv_lens) - out).max() > 1e-3


def test_placement_and_poison_invariance():
    lens = np.array([1, 15, 16, 17, 100, 255], dtype=np.int32)
    clean = wl.make_paged_batch(lens, 4, 2, 32, dtype="fp32", seed=21, spare_blocks=4)
    ref = oa.decode_attention(clean.q, clean.k_blocks, clean.v_blocks, clean.block_table, clean.kv_lens)
    moved = wl.repage(clean, seed=99)
    assert not np.array_equal(moved.block_table, clean.block_table)
    np.testing.assert_array_equal(
        oa.decode_attention(moved.q, moved.k_blocks, moved.v_blocks, moved.block_table, moved.kv_lens), ref)
    for kind in ("nan", "inf", "ninf", "big"):
        p = wl.make_paged_batch(lens, 4, 2, 32, dtype="fp32", seed=21, spare_blocks=4, poison=kind)
        np.testing.assert_array_equal(
            oa.decode_attention(p.q, p.k_blocks, p.v_blocks, p.block_table, p.kv_lens), ref)


def test_split_merge_identity():
    rng = np.random.default_rng(13)
    L, D = 101, 24
    K, V, q = rng.standard_normal((L, D)), rng.standard_normal((L, D)), rng.standard_normal(D)
    sc = 1 / math.sqrt(D)
    full = oa.attention_single(q, K, V, sc)
    for cuts in ([0, 101], [0, 50, 101], [0, 1, 17, 64, 101], list(range(0, 102))):
        ms, ls, accs = [], [], []
        for a, b in zip(cuts[:-1], cuts[1:]):
            s = (K[a:b] @ q) * sc
            m = s.max()
            p = np.exp(s - m)
            ms.append(m); ls.append(p.sum()); accs.append(p @ V[a:b])
        np.testing.assert_allclose(oa.merge_partials(ms, ls, accs), full, atol=1e-13)


def test_bf16_inputs_are_exact_in_the_oracle():
    # bf16 bit patterns widen exactly; oracle on widened values == oracle on
    # the same values stored as float64
    pb = wl.make_paged_batch(np.array([33, 70], dtype=np.int32), 2, 1, 64, dtype="bf16", seed=3)
    q, k, v = pb.as_float("q"), pb.as_float("k_blocks"), pb.as_float("v_blocks")
    assert q.dtype == np.float32
    a = oa.decode_attention(q, k, v, pb.block_table, pb.kv_lens)
    b = oa.decode_attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64),
                            pb.block_table, pb.kv_lens)
    np.testing.assert_array_equal(a, b)


def test_rejects_empty_kv():
    pb = wl.make_paged_batch(np.array([4], dtype=np.int32), 1, 1, 8, dtype="fp32")
    with pytest.raises(ValueError):
        oa.decode_attention(pb.q, pb.k_blocks, pb.v_blocks, pb.block_table, np.array([0]))
