"""GPU tests of KV staging (host pool -> HBM pool), the reverse move, and the
copy/compute handshake of the double-buffered pool."""
import numpy as np
import pytest

from paper_2605_23389_amd import workloads as wl
from tests.gpu_util import check_parity, oracle_out

pytestmark = pytest.mark.gpu


def _pinned(shape, dtype):
    import torch
    return torch.empty(shape, dtype=dtype, pin_memory=True)


def test_stage_is_byte_exact_and_leaves_other_slots_alone(lib):
    import torch
    rng = np.random.default_rng(0)
    block_bytes = 8 * 16 * 128 * 2          # one GQA block (8 KV heads, bf16)
    n_host, n_dev = 64, 48
    hk, hv = _pinned((n_host, block_bytes), torch.uint8), _pinned((n_host, block_bytes), torch.uint8)
    hk.copy_(torch.from_numpy(rng.integers(0, 256, (n_host, block_bytes), dtype=np.uint8)))
    hv.copy_(torch.from_numpy(rng.integers(0, 256, (n_host, block_bytes), dtype=np.uint8)))
    dk = torch.full((n_dev, block_bytes), 0xAB, dtype=torch.uint8, device="cuda")
    dv = torch.full((n_dev, block_bytes), 0xCD, dtype=torch.uint8, device="cuda")
    # runs of consecutive ids, single blocks, and a reversed stretch
    src = np.array([3, 4, 5, 6, 40, 10, 11, 63, 20, 19, 18], dtype=np.int64)
    dst = np.array([7, 8, 9, 10, 0, 30, 31, 47, 12, 13, 14], dtype=np.int32)
    s = torch.cuda.Stream()
    lib.stage_kv(hk, hv, src, dk, dv, dst, block_bytes, stream=s)
    s.synchronize()
    dk_h, dv_h = dk.cpu().numpy(), dv.cpu().numpy()
    for a, b in zip(src, dst):
        assert np.array_equal(dk_h[b], hk.numpy()[a]) and np.array_equal(dv_h[b], hv.numpy()[a])
    untouched = sorted(set(range(n_dev)) - set(dst.tolist()))
    assert (dk_h[untouched] == 0xAB).all() and (dv_h[untouched] == 0xCD).all()
    # K only
    dk.fill_(0)
    lib.stage_kv(hk, None, src[:3], dk, None, dst[:3], block_bytes, stream=s)
    s.synchronize()
    assert np.array_equal(dk[7:10].cpu().numpy(), hk.numpy()[3:6])

    # the reverse move restores the host blocks
    hk2, hv2 = _pinned((n_host, block_bytes), torch.uint8), _pinned((n_host, block_bytes), torch.uint8)
    hk2.zero_(); hv2.zero_()
    lib.stage_kv(hk, hv, src, dk, dv, dst, block_bytes, stream=s)
    lib.unstage_kv(hk2, hv2, src, dk, dv, dst, block_bytes, stream=s)
    s.synchronize()
    for a in src:
        assert np.array_equal(hk2.numpy()[a], hk.numpy()[a]) and np.array_equal(hv2.numpy()[a], hv.numpy()[a])
    rest = sorted(set(range(n_host)) - set(src.tolist()))
    assert (hk2.numpy()[rest] == 0).all()


def test_stage_rejects_unpinned_host_memory(lib):
    import torch
    from paper_2605_23389_amd import binding as als
    hk = torch.zeros((4, 4096), dtype=torch.uint8)          # pageable
    dk = torch.zeros((4, 4096), dtype=torch.uint8, device="cuda")
    with pytest.raises(als.AlignedServeError) as e:
        lib.stage_kv(hk, None, [0], dk, None, [0], 4096)
    assert e.value.status == als.AS_EINVAL and "pinned" in str(e.value)
    # the failed check leaves no sticky error behind
    torch.cuda.synchronize()
    assert int(dk.sum()) == 0


def _host_pool_from(pb):
    """Pinned host copies of a PagedBatch's pools (bf16 carried as int16)."""
    import torch
    hk = _pinned(pb.k_blocks.shape, torch.int16)
    hv = _pinned(pb.v_blocks.shape, torch.int16)
    hk.copy_(torch.from_numpy(pb.k_blocks.view(np.int16)))
    hv.copy_(torch.from_numpy(pb.v_blocks.view(np.int16)))
    return hk, hv


def test_attention_on_staged_blocks_is_bitwise_the_same(lib):
    import torch
    lens = wl.uniform_lengths(np.random.default_rng(2), 6, 20, 700)
    pb = wl.make_paged_batch(lens, 8, 2, 128, dtype="bf16", seed=2, spare_blocks=1)
    hk, hv = _host_pool_from(pb)
    NB = pb.num_blocks
    block_bytes = 2 * 16 * 128 * 2
    # direct initialisation
    dk0 = hk.cuda().view(torch.bfloat16)
    dv0 = hv.cuda().view(torch.bfloat16)
    bt0 = torch.from_numpy(pb.block_table).cuda()
    q = torch.from_numpy(pb.q.view(np.int16)).cuda().view(torch.bfloat16)
    dl = torch.from_numpy(pb.kv_lens).cuda()
    out0 = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    lib.decode_attention(q, dk0, dv0, bt0, dl, out0, kv_lens_host=pb.kv_lens)
    # staged into a larger poisoned pool at shuffled slots
    slots = np.random.default_rng(3).permutation(NB + 5)[:NB].astype(np.int32)   # host id i -> slot
    dk1 = torch.full((NB + 5,) + tuple(pb.k_blocks.shape[1:]), float("nan"), dtype=torch.bfloat16, device="cuda")
    dv1 = torch.full_like(dk1, float("nan"))
    side = torch.cuda.Stream()
    lib.stage_kv(hk, hv, np.arange(NB, dtype=np.int64), dk1, dv1, slots, block_bytes, stream=side)
    side.synchronize()
    bt1 = torch.from_numpy(slots[pb.block_table]).cuda()
    out1 = torch.empty_like(out0)
    lib.decode_attention(q, dk1, dv1, bt1, dl, out1, kv_lens_host=pb.kv_lens)
    torch.cuda.synchronize()
    assert torch.equal(out0, out1)
    check_parity(out1.double().cpu().numpy(), oracle_out(pb), pb, out_dtype="fp32")


def test_double_buffered_pipeline_orders_copies_and_attention(lib):
    """Stage batch i+1 on the side stream while batch i is attended on the
    compute stream, two buffers, with the side stream artificially slowed so
    that a missing wait would read poisoned blocks."""
    import torch
    from paper_2605_23389_amd import binding as als
    Hq, Hkv, D = 8, 2, 128
    block_bytes = Hkv * 16 * D * 2
    rng = np.random.default_rng(7)
    batches = [wl.make_paged_batch(wl.uniform_lengths(rng, 4, 30, 500), Hq, Hkv, D, dtype="bf16",
                                   seed=100 + i) for i in range(5)]
    refs = [oracle_out(pb) for pb in batches]
    cap = max(pb.num_blocks for pb in batches)
    pool_k = torch.full((2 * cap, Hkv, 16, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    pool_v = torch.full_like(pool_k, float("nan"))
    hosts = [_host_pool_from(pb) for pb in batches]
    pipe = als.Pipeline(2)
    side = torch.cuda.ExternalStream(pipe.stream)
    compute = torch.cuda.Stream()
    outs = []

    def stage(i):
        buf = i % 2
        pb = batches[i]
        pipe.begin_stage(buf)
        with torch.cuda.stream(side):
            torch.cuda._sleep(20_000_000)            # a few ms: copies start late
        dst = (np.arange(pb.num_blocks) + buf * cap).astype(np.int32)
        lib.stage_kv(hosts[i][0], hosts[i][1], np.arange(pb.num_blocks, dtype=np.int64), pool_k, pool_v,
                     dst, block_bytes, stream=pipe.stream)
        pipe.end_stage(buf)

    stage(0)
    for i, pb in enumerate(batches):
        buf = i % 2
        if i + 1 < len(batches):
            stage(i + 1)                              # overlaps with attention of batch i
        pipe.acquire(buf, stream=compute)
        with torch.cuda.stream(compute):
            q = torch.from_numpy(pb.q.view(np.int16)).cuda().view(torch.bfloat16)
            bt = torch.from_numpy(pb.block_table + buf * cap).cuda()
            dl = torch.from_numpy(pb.kv_lens).cuda()
            out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
            lib.decode_attention(q, pool_k, pool_v, bt, dl, out, kv_lens_host=pb.kv_lens, stream=compute)
            # poison the buffer after use: the next stage into it must wait for this
            pool_k[buf * cap:(buf + 1) * cap].fill_(float("nan"))
            pool_v[buf * cap:(buf + 1) * cap].fill_(float("nan"))
        pipe.release(buf, stream=compute)
        outs.append(out)
    torch.cuda.synchronize()
    pipe.destroy()
    for out, ref, pb in zip(outs, refs, batches):
        check_parity(out.double().cpu().numpy(), ref, pb, out_dtype="fp32")


@pytest.mark.parametrize("policy", ["auto", "dma", "kernel"])
@pytest.mark.parametrize("block_bytes", [32768, 16384 + 4096 + 48, 4096, 131072])
def test_stage_paths_agree_byte_for_byte(lib, policy, block_bytes):
    """Every way of moving the blocks (DMA copies per run, the gather kernel,
    or the automatic choice) leaves the same bytes in the same slots, in both
    directions, for block sizes with and without a ragged last part, and for
    more blocks than one kernel launch carries ids for."""
    import torch
    from paper_2605_23389_amd import binding as als
    rng = np.random.default_rng(block_bytes)
    n_host, n_dev, m = 700, 640, 600
    hk, hv = _pinned((n_host, block_bytes), torch.uint8), _pinned((n_host, block_bytes), torch.uint8)
    hk.copy_(torch.from_numpy(rng.integers(0, 256, (n_host, block_bytes), dtype=np.uint8)))
    hv.copy_(torch.from_numpy(rng.integers(0, 256, (n_host, block_bytes), dtype=np.uint8)))
    dk = torch.full((n_dev, block_bytes), 0xAB, dtype=torch.uint8, device="cuda")
    dv = torch.full((n_dev, block_bytes), 0xCD, dtype=torch.uint8, device="cuda")
    src = rng.permutation(n_host)[:m].astype(np.int64)      # scattered: runs of one block
    dst = rng.permutation(n_dev)[:m].astype(np.int32)
    src[100:140] = np.arange(300, 340)                      # plus one long run (may repeat earlier ids: reads only)
    dst_run = np.setdiff1d(np.arange(n_dev), np.delete(dst, np.s_[100:140]))[:40]
    assert len(dst_run) == 40 and np.all(np.diff(dst_run) >= 1)
    dst[100:140] = dst_run
    assert len(set(dst.tolist())) == m
    s = torch.cuda.Stream()
    als.stage_set_policy({"auto": als.STAGE_AUTO, "dma": als.STAGE_DMA, "kernel": als.STAGE_KERNEL}[policy])
    try:
        lib.stage_kv(hk, hv, src, dk, dv, dst, block_bytes, stream=s)
        s.synchronize()
        dk_h, dv_h = dk.cpu().numpy(), dv.cpu().numpy()
        assert np.array_equal(dk_h[dst], hk.numpy()[src]) and np.array_equal(dv_h[dst], hv.numpy()[src])
        untouched = np.setdiff1d(np.arange(n_dev), dst)
        assert (dk_h[untouched] == 0xAB).all() and (dv_h[untouched] == 0xCD).all()
        # eviction: device -> distinct host slots
        hk2 = _pinned((n_host, block_bytes), torch.uint8); hk2.zero_()
        hdst = rng.permutation(n_host)[:m].astype(np.int64)
        lib.unstage_kv(hk2, None, hdst, dk, None, dst, block_bytes, stream=s)
        s.synchronize()
        assert np.array_equal(hk2.numpy()[hdst], dk_h[dst])
        rest = np.setdiff1d(np.arange(n_host), hdst)
        assert (hk2.numpy()[rest] == 0).all()
    finally:
        als.stage_set_policy(als.STAGE_AUTO)


def test_stage_policy_rejects_unknown_value(lib):
    from paper_2605_23389_amd import binding as als
    with pytest.raises(als.AlignedServeError):
        als.stage_set_policy(7)


def test_pipeline_query_follows_the_copies(lib):
    """as_pipeline_query polls a buffer's "ready" event from the host: complete before anything
    was staged, not complete while the side stream is still busy ahead of the copies, complete
    after they have finished -- and it never blocks."""
    import time
    import torch
    from paper_2605_23389_amd import binding as als
    block_bytes = 4096
    host = _pinned((8, block_bytes), torch.uint8)
    host.copy_(torch.arange(8 * block_bytes, dtype=torch.int64).remainder(251).to(torch.uint8).view(8, block_bytes))
    dev = torch.zeros((8, block_bytes), dtype=torch.uint8, device="cuda")
    pipe = als.Pipeline(2)
    side = torch.cuda.ExternalStream(pipe.stream)
    assert pipe.query(0) and pipe.query(1)                 # nothing staged yet
    pipe.begin_stage(1)
    with torch.cuda.stream(side):
        torch.cuda._sleep(400_000_000)                     # keeps the side stream busy for a while
    lib.stage_kv(host, None, np.arange(8, dtype=np.int64), dev, None, np.arange(8, dtype=np.int32), block_bytes,
                 stream=pipe.stream)
    pipe.end_stage(1)
    t0 = time.perf_counter()
    early = pipe.query(1)
    assert time.perf_counter() - t0 < 0.05                 # a poll, not a wait
    assert not early
    assert pipe.query(0)                                   # the other buffer is unaffected
    side.synchronize()
    assert pipe.query(1)
    assert torch.equal(dev.cpu(), host)
    with pytest.raises(als.AlignedServeError):
        pipe.query(2)
    pipe.destroy()
