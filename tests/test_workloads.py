"""The seeded input generators: representation helpers and config recipes."""
import numpy as np

from paper_2605_23389_amd import workloads as wl


def test_bf16_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.3895313892515355e38], dtype=np.float32)
    b = wl.f32_to_bf16_bits(x)
    # 1.00390625 = 1 + 2^-8 is a tie between 1.0 and 1+2^-7 -> even (1.0)
    assert b[0] == 0x3F80 and b[1] == 0x3F80
    # 1.01171875 = 1 + 3*2^-8 is a tie between 1+2^-7 and 1+2^-6 -> even (1+2^-6)
    assert b[2] == 0x3F82
    assert wl.bf16_bits_to_f32(b)[3] == -2.5
    assert b[4] == 0
    back = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.float32([0.1, -7.7, 1e-3])))
    assert np.all(np.abs(back - np.float32([0.1, -7.7, 1e-3])) <= np.abs(np.float32([0.1, -7.7, 1e-3])) * 2.0 ** -8)
    assert np.isnan(wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.float32([np.nan]))))[0]
    # torch agrees
    import torch
    r = np.random.default_rng(0).standard_normal(4096, dtype=np.float32)
    t = torch.from_numpy(r).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(t, wl.f32_to_bf16_bits(r))


def test_config_lengths_match_recipe():
    l1 = wl.config_lengths(1)
    assert l1.shape == (64,) and l1.min() >= 128 and l1.max() <= 8192
    l2 = wl.config_lengths(2)
    assert l2.shape == (1024,) and l2.min() >= 64 and l2.max() <= 32768
    l3 = wl.config_lengths(3)
    assert l3.shape == (128,) and l3.min() >= 4096 and l3.max() <= 32768
    assert np.array_equal(wl.config_lengths(2, seed=0), l2)
    assert not np.array_equal(wl.config_lengths(2, seed=1), l2)
    assert abs(np.median(wl.config_lengths(4)) - 2048) < 150


def test_paged_batch_layout_and_poison():
    lens = np.array([1, 16, 17, 40], dtype=np.int32)
    pb = wl.make_paged_batch(lens, 4, 2, 8, dtype="bf16", seed=1, spare_blocks=2, poison="nan")
    assert pb.k_blocks.shape == (1 + 1 + 2 + 3 + 2, 2, 16, 8) and pb.k_blocks.dtype == np.uint16
    kf = pb.as_float("k_blocks")
    used = set()
    for b in range(4):
        nb = (lens[b] + 15) // 16
        ids = pb.block_table[b, :nb].tolist()
        assert not (used & set(ids))
        used |= set(ids)
        tail = lens[b] % 16
        if tail:
            assert np.isnan(kf[ids[-1], :, tail:, :]).all()
            assert np.isfinite(kf[ids[-1], :, :tail, :]).all()
    spare = set(range(pb.num_blocks)) - used
    assert len(spare) == 2 and all(np.isnan(kf[s]).all() for s in spare)
    assert set(pb.block_table[0, 1:].tolist()) <= spare


def test_random_grouping_and_block_table():
    order, offs = wl.random_grouping(10, 4, seed=3)
    assert sorted(order.tolist()) == list(range(10)) and offs.tolist() == [0, 4, 8, 10]
    bt, used = wl.build_block_table([16, 17, 1], seed=0, num_blocks=10)
    assert used == 4 and bt.shape == (3, 2)
    ids = [bt[0, 0], bt[1, 0], bt[1, 1], bt[2, 0]]
    assert len(set(ids)) == 4 and max(ids) < 10


def test_fp16_bits_round_to_nearest_even_and_widen_exactly():
    # 1 + 2^-11 is a tie between 1 and 1 + 2^-10: goes to the even mantissa (1.0);
    # 1 + 3*2^-11 is a tie that goes up to 1 + 2^-9
    x = np.float32([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, -2.5, 65520.0, 6e-8])
    b = wl.f32_to_f16_bits(x)
    assert b.dtype == np.uint16
    assert b[0] == 0x3C00 and b[1] == 0x3C02 and b[2] == 0xC100
    assert b[3] == 0x7C00            # rounds to +inf (largest finite is 65504)
    assert b[4] == 0x0001            # smallest subnormal, 2^-24
    back = wl.f16_bits_to_f32(b[:3])
    assert back.tolist() == [1.0, 1.0 + 2.0 ** -9, -2.5]
    pb = wl.make_paged_batch(np.array([5, 20], dtype=np.int32), 4, 2, 8, dtype="fp16", seed=1)
    assert pb.q.dtype == np.uint16
    q = pb.as_float("q")
    assert np.array_equal(wl.f32_to_f16_bits(q), pb.q)      # already representable
